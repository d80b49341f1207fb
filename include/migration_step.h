/*
 * migration_step.h — C ABI of one scheduling decision of the progress-aware workload
 * migration (host code only; no GPU work).
 *
 * Section 6.3, Algorithm 1: for every PP stage i and time slot the Scheduler computes the
 * progress P_d of every DP group d at that stage (forward workloads completed, local and
 * migrated), takes d_min = argmin_d P_d and d_max = argmax_d P_d, and, if (d_min, i) is
 * fail-stop or P_dmax - P_dmin > delta, moves the next pending micro-batch of d_min at this
 * stage to d_max, provided the destination can hold it (memory).
 * Readings: a fail-stop group is never a destination and is the source while it has pending
 * work (lowest index first); ties of argmin / argmax go to the lowest index; a group is not
 * its own destination.  The pipeline advance around this step is not part of this library.
 *
 * All pointers are HOST pointers owned by the caller.
 */
#ifndef MIGRATION_STEP_H_
#define MIGRATION_STEP_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIGRATION_STEP_NONE 0         /* nothing moves in this slot */
#define MIGRATION_STEP_MIGRATE 1      /* *source, *destination, *micro_batch are set */
#define MIGRATION_STEP_INVALID_ARG (-1)

#define MIGRATION_STEP_NO_PENDING (-1) /* value of next_pending[d] when group d has none */

/* progress: P_d for the num_groups DP groups at this stage; fail_stop: non-zero = the stage of
 * group d has crashed; delta: progress-imbalance threshold (>= 0); next_pending: id of the next
 * pending micro-batch of group d at this stage or MIGRATION_STEP_NO_PENDING; memory_feasible:
 * non-zero = the stage of group d could hold one more migrated micro-batch. */
int migration_step_decide(const int32_t* progress, const uint8_t* fail_stop, int32_t num_groups,
                          int32_t delta, const int32_t* next_pending,
                          const uint8_t* memory_feasible, int32_t* source, int32_t* destination,
                          int32_t* micro_batch);

#ifdef __cplusplus
}
#endif
#endif /* MIGRATION_STEP_H_ */
