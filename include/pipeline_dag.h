/*
 * pipeline_dag.h — C ABI of the iteration-time predictor (host code only; no GPU work).
 *
 * Section 5.2, "Iteration-time Prediction": the pipeline schedule is a DAG whose vertices are
 * the computation chunks F(m,s), B(m,s), W(m,s) (forward, backward-activation, backward-weight
 * of micro-batch m at stage s) with their execution costs.  Data edges F(m,s-1) -> F(m,s) and
 * B(m,s+1) -> B(m,s) carry the point-to-point time; F(m,S-1) -> B(m,S-1), F(m,s) -> B(m,s) and
 * B(m,s) -> W(m,s) carry none; consecutive chunks of one stage, in the order of the schedule,
 * are joined by zero-weight resource edges.  Earliest start times follow
 *     t_start(v) = max over predecessors u of  t_start(u) + cost(u) + edge(u, v)      (Eq. 2)
 * and the predicted healthy iteration time is the completion time of the last vertex.
 *
 * All pointers are HOST pointers owned by the caller; the calls allocate only transient host
 * memory and keep nothing.
 */
#ifndef PIPELINE_DAG_H_
#define PIPELINE_DAG_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PIPELINE_DAG_OK 0
#define PIPELINE_DAG_INVALID_ARG (-1)   /* null pointer, non-positive size, bad kind or index */
#define PIPELINE_DAG_BAD_SCHEDULE (-2)  /* a chunk twice or missing, or an order that
                                           contradicts the data dependencies */

#define PIPELINE_DAG_F 0
#define PIPELINE_DAG_B 1
#define PIPELINE_DAG_W 2

typedef struct {
  int32_t kind;       /* PIPELINE_DAG_F / _B / _W */
  int32_t microbatch; /* 0 .. microbatches - 1 */
} pipeline_dag_chunk;

/* Chunk orders of the two schedules of Table 3.  `order` holds stages * per_stage entries,
 * stage-major; per_stage = 2 * microbatches (1F1B: the backward is one chunk, kinds F and B)
 * or 3 * microbatches (ZB-H1: B and W split).
 * 1F1B: stage s runs min(S-1-s, M) warm-up forwards, alternates one forward and one backward,
 * then drains the backwards.  ZB-H1 (same activation memory as 1F1B): at every unit-cost time
 * step a stage runs a ready B if there is one, else a ready F if fewer than S-s micro-batches
 * are in flight on it, else a pending W. */
int pipeline_dag_schedule_1f1b(int32_t stages, int32_t microbatches, pipeline_dag_chunk* order);
int pipeline_dag_schedule_zbh1(int32_t stages, int32_t microbatches, pipeline_dag_chunk* order);

/* Eq. 2 over a schedule.  kinds = 2 (F, B) or 3 (F, B, W); order: stages * kinds *
 * microbatches entries, stage-major, every chunk of a stage exactly once; cost: fp64
 * [kinds][microbatches][stages], cost >= 0; p2p >= 0.  Writes the iteration time and, if
 * t_start is not NULL, the start times in the layout of cost. */
int pipeline_dag_simulate(int32_t stages, int32_t microbatches, int32_t kinds,
                          const pipeline_dag_chunk* order, const double* cost, double p2p,
                          double* iteration_time, double* t_start);

#ifdef __cplusplus
}
#endif
#endif /* PIPELINE_DAG_H_ */
