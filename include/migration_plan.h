/*
 * migration_plan.h — C ABI of the progress-aware workload migration loop (host code only).
 *
 * Section 6.3, Algorithm 1: while unfinished workloads exist, the Scheduler advances the
 * pipeline schedules of all DP groups by one time slot and then, for every PP stage, takes one
 * migration decision (migration_step.h) from the progress P_{d,i,t} of the groups at that stage.
 * The objective of the section's problem statement is the largest completion time over the DP
 * groups; its constraints are that every stage of every micro-batch runs exactly once, that
 * dependencies survive a move, and that the activations held by a stage never exceed its
 * capacity (they live until the corresponding backward completes).
 *
 * The time slots, the pipeline advance and the memory accounting are shown in a figure only;
 * this library fixes them as follows.  Every (group, stage) is an executor that runs one chunk
 * at a time.  Chunks are the forward F and the backward B of a micro-batch at a stage (the
 * weight-gradient chunk W follows its B on the same executor and has no successor: its time is
 * part of B's).  F at stage i needs F at stage i - 1; B at stage i needs B at stage i + 1 (the
 * last stage: its own F) and runs where the F of that stage ran; across stages a chunk becomes
 * ready `p2p` slots after its predecessor completed.  An idle executor starts a ready B if it
 * has one (lowest source group, then lowest micro-batch), else the first ready F of its queue
 * provided it holds fewer than `capacity` activations (forwards started whose backward has not
 * completed), else nothing.  A queue holds the group's own micro-batches in order and migrated
 * ones behind them.  A fail-stop stage is known from the start and runs nothing.  The next
 * pending micro-batch of a group at a stage is the first forward of its queue that has not
 * started; a destination is memory-feasible if it holds fewer than `capacity` activations at
 * the slot of the decision; after a move the source's progress counts one forward more (it has
 * one fewer to do) and the destination's when it completes the forward.  The completion time of
 * a group is the last slot in which one of its executors completes a chunk.
 *
 * All pointers are HOST pointers owned by the caller; two-dimensional arrays are row-major
 * [group][stage], `assignment` and `executed` are [group][micro_batch][stage].
 */
#ifndef MIGRATION_PLAN_H_
#define MIGRATION_PLAN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIGRATION_PLAN_OK 0
#define MIGRATION_PLAN_INVALID_ARG (-1)
#define MIGRATION_PLAN_UNSCHEDULABLE (-2)   /* some workload can never run (e.g. a stage is fail-stop
                                               in every group); outputs are undefined */
#define MIGRATION_PLAN_MOVES_OVERFLOW (-3)  /* more moves than moves_capacity; outputs are undefined */

/* One migration: at `slot`, the stage-`stage` workload of micro-batch `micro_batch` of source
 * group `group` left the queue of `source` for the queue of `destination`. */
typedef struct {
  int32_t slot, stage, source, destination, group, micro_batch;
} migration_plan_move;

/* Runs the loop until every chunk has completed.
 * f_cost, b_cost: slots per F / B chunk on every executor (>= 1); fail_stop: non-zero = the stage
 * has crashed; capacity: activations a stage can hold (>= 1); delta: progress-imbalance
 * threshold (>= 0); p2p: slots between stages (>= 0); migrate: 0 = take no decisions (the
 * schedule as it would run untouched).
 * assignment: NULL, or the executor group of every workload (then no decisions are taken): the
 * form a search over static plans uses.
 * Outputs: makespan[group]; executed[group][micro_batch][stage] = executor group; up to
 * moves_capacity moves in decision order and their number; the iteration time (largest makespan).
 * makespan, executed, moves may be NULL (moves_capacity is then taken as unlimited and only the
 * count is returned). */
int migration_plan_run(int32_t n_groups, int32_t n_stages, int32_t n_micro, const int32_t* f_cost,
                       const int32_t* b_cost, const uint8_t* fail_stop, const int32_t* capacity,
                       int32_t delta, int32_t p2p, int32_t migrate, const int32_t* assignment,
                       int32_t* makespan, int32_t* executed, migration_plan_move* moves,
                       int32_t moves_capacity, int32_t* n_moves, int32_t* iteration_time);

#ifdef __cplusplus
}
#endif
#endif /* MIGRATION_PLAN_H_ */
