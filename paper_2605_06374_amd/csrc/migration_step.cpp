// One scheduling decision of Algorithm 1 (Section 6.3): host code, a single pass over the
// DP groups.
#include "migration_step.h"

extern "C" int migration_step_decide(const int32_t* progress, const uint8_t* fail_stop,
                                     int32_t n, int32_t delta, const int32_t* next_pending,
                                     const uint8_t* memory_feasible, int32_t* source,
                                     int32_t* destination, int32_t* micro_batch) {
  if (!progress || !fail_stop || !next_pending || !memory_feasible || !source || !destination ||
      !micro_batch || n < 1 || delta < 0)
    return MIGRATION_STEP_INVALID_ARG;
  int d_max = -1, d_min = -1, evict = -1;
  for (int d = 0; d < n; ++d) {
    if (fail_stop[d]) {
      if (evict < 0 && next_pending[d] != MIGRATION_STEP_NO_PENDING) evict = d;
      continue;
    }
    if (d_max < 0 || progress[d] > progress[d_max]) d_max = d;   // first of the largest
    if (d_min < 0 || progress[d] < progress[d_min]) d_min = d;   // first of the smallest
  }
  if (d_max < 0) return MIGRATION_STEP_NONE;                      // no healthy group left
  int src = evict;
  if (src < 0) {
    if (!(progress[d_max] - progress[d_min] > delta)) return MIGRATION_STEP_NONE;
    src = d_min;
  }
  if (src == d_max || next_pending[src] == MIGRATION_STEP_NO_PENDING || !memory_feasible[d_max])
    return MIGRATION_STEP_NONE;
  *source = src;
  *destination = d_max;
  *micro_batch = next_pending[src];
  return MIGRATION_STEP_MIGRATE;
}
