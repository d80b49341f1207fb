// The loop of Algorithm 1 (Section 6.3) around a slot-by-slot simulation of the pipelines of all
// DP groups: host code.  The rules are stated in migration_plan.h; the decision inside the loop
// is migration_step_decide.
#include "migration_plan.h"

#include <algorithm>
#include <utility>
#include <vector>

#include "migration_step.h"

namespace {

struct Work { int32_t d, j; };
inline bool operator<(const Work& a, const Work& b) { return a.d != b.d ? a.d < b.d : a.j < b.j; }

struct Executor {
  std::vector<Work> queue;    // forwards assigned here that have not started, in order
  std::vector<Work> owed_b;   // backwards still to run here (their forward completed here)
  int32_t busy_until = 0, live = 0, progress = 0;
  int running = 0;            // 0 idle, 1 forward, 2 backward
  Work work{0, 0};
};

}  // namespace

extern "C" int migration_plan_run(int32_t D, int32_t I, int32_t M, const int32_t* f_cost,
                                  const int32_t* b_cost, const uint8_t* fail_stop,
                                  const int32_t* capacity, int32_t delta, int32_t p2p,
                                  int32_t migrate, const int32_t* assignment, int32_t* makespan,
                                  int32_t* executed, migration_plan_move* moves,
                                  int32_t moves_capacity, int32_t* n_moves,
                                  int32_t* iteration_time) {
  if (D < 1 || I < 1 || M < 1 || !f_cost || !b_cost || !fail_stop || !capacity || delta < 0 ||
      p2p < 0 || !n_moves || !iteration_time || (moves && moves_capacity < 0))
    return MIGRATION_PLAN_INVALID_ARG;
  if ((int64_t)D * I * M > (1 << 26)) return MIGRATION_PLAN_INVALID_ARG;
  int32_t worst = 0;
  for (int x = 0; x < D * I; ++x) {
    if (f_cost[x] < 1 || b_cost[x] < 1 || capacity[x] < 1) return MIGRATION_PLAN_INVALID_ARG;
    worst = std::max(worst, f_cost[x] + b_cost[x]);
  }
  if (assignment) {
    migrate = 0;
    for (int64_t x = 0; x < (int64_t)D * M * I; ++x)
      if (assignment[x] < 0 || assignment[x] >= D) return MIGRATION_PLAN_INVALID_ARG;
  }
  const int64_t max_slots = 4ll * D * M * I * (worst + p2p) + 1000;
  auto at = [&](int e, int i) { return e * I + i; };
  auto wk = [&](int d, int j, int i) { return ((int64_t)d * M + j) * I + i; };
  std::vector<Executor> ex((size_t)D * I);
  for (int d = 0; d < D; ++d)
    for (int j = 0; j < M; ++j)
      for (int i = 0; i < I; ++i)
        ex[at(assignment ? assignment[wk(d, j, i)] : d, i)].queue.push_back(Work{d, j});
  std::vector<int32_t> done_f((size_t)D * M * I, -1), done_b((size_t)D * M * I, -1);
  std::vector<int32_t> span(D, 0);
  std::vector<int32_t> progress(D), next_pending(D);
  std::vector<uint8_t> stopped(D), feasible(D);
  int64_t remaining = 2ll * D * M * I;
  int32_t count = 0;
  for (int64_t t = 0; remaining > 0; ++t) {
    if (t > max_slots) return MIGRATION_PLAN_UNSCHEDULABLE;
    // ---- advance the pipeline schedules: completions of this slot ...
    for (int e = 0; e < D; ++e)
      for (int i = 0; i < I; ++i) {
        Executor& x = ex[at(e, i)];
        if (!x.running || x.busy_until != t) continue;
        span[e] = (int32_t)t;
        if (x.running == 1) {
          done_f[wk(x.work.d, x.work.j, i)] = (int32_t)t;
          x.progress += 1;
          x.owed_b.push_back(x.work);
        } else {
          done_b[wk(x.work.d, x.work.j, i)] = (int32_t)t;
          x.live -= 1;
        }
        x.running = 0;
        --remaining;
      }
    // ... then every idle executor starts what it can
    for (int e = 0; e < D; ++e)
      for (int i = 0; i < I; ++i) {
        Executor& x = ex[at(e, i)];
        if (x.running || fail_stop[at(e, i)]) continue;
        int pick = -1;
        // a ready backward first: lowest (group, micro-batch)
        for (size_t n = 0; n < x.owed_b.size(); ++n) {
          const Work w = x.owed_b[n];
          const int32_t pred = i == I - 1 ? done_f[wk(w.d, w.j, i)] : done_b[wk(w.d, w.j, i + 1)];
          if (pred < 0 || pred + (i == I - 1 ? 0 : p2p) > t) continue;
          if (pick < 0 || w < x.owed_b[pick]) pick = (int)n;
        }
        if (pick >= 0) {
          x.work = x.owed_b[pick];
          x.owed_b.erase(x.owed_b.begin() + pick);
          x.running = 2;
          x.busy_until = (int32_t)t + b_cost[at(e, i)];
          continue;
        }
        if (x.live >= capacity[at(e, i)]) continue;
        // else the first ready forward of the queue
        for (size_t n = 0; n < x.queue.size(); ++n) {
          const Work w = x.queue[n];
          if (i > 0) {
            const int32_t pred = done_f[wk(w.d, w.j, i - 1)];
            if (pred < 0 || pred + p2p > t) continue;
          }
          pick = (int)n;
          break;
        }
        if (pick < 0) continue;
        x.work = x.queue[pick];
        x.queue.erase(x.queue.begin() + pick);
        if (executed) executed[wk(x.work.d, x.work.j, i)] = e;
        x.live += 1;
        x.running = 1;
        x.busy_until = (int32_t)t + f_cost[at(e, i)];
      }
    // ---- one decision per stage
    if (!migrate) continue;
    for (int i = 0; i < I; ++i) {
      for (int e = 0; e < D; ++e) {
        const Executor& x = ex[at(e, i)];
        progress[e] = x.progress;
        stopped[e] = fail_stop[at(e, i)];
        next_pending[e] = x.queue.empty() ? MIGRATION_STEP_NO_PENDING : x.queue[0].d * M + x.queue[0].j;
        feasible[e] = x.live < capacity[at(e, i)];
      }
      int32_t src, dst, mb;
      const int rc = migration_step_decide(progress.data(), stopped.data(), D, delta,
                                           next_pending.data(), feasible.data(), &src, &dst, &mb);
      if (rc != MIGRATION_STEP_MIGRATE) continue;
      Executor& from = ex[at(src, i)];
      const Work w = from.queue[0];
      from.queue.erase(from.queue.begin());
      ex[at(dst, i)].queue.push_back(w);
      from.progress += 1;
      if (moves) {
        if (count >= moves_capacity) return MIGRATION_PLAN_MOVES_OVERFLOW;
        moves[count] = migration_plan_move{(int32_t)t, i, src, dst, w.d, w.j};
      }
      ++count;
    }
  }
  int32_t longest = 0;
  for (int d = 0; d < D; ++d) {
    if (makespan) makespan[d] = span[d];
    longest = std::max(longest, span[d]);
  }
  *n_moves = count;
  *iteration_time = longest;
  return MIGRATION_PLAN_OK;
}
