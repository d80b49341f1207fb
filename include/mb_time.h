/*
 * mb_time.h — C ABI of the micro-batch time predictor (host code only; no GPU work).
 *
 * Section 5.2, "Micro-Batch Time Prediction": the execution time of a packed micro-batch with
 * documents l_1..l_k, sum N, is modelled as
 *     T_MB ~ alpha * N + beta * sum_i l_i^2                                     (Eq. 1)
 * with alpha and beta profiled during a warm-up phase (here: fitted by least squares to
 * measured times).  At the end of Section 5.2 a change point whose observed time exceeds the
 * predicted healthy time by more than 25 % goes on to validation; otherwise it is benign.
 *
 * All pointers are HOST pointers owned by the caller; nothing is allocated or kept.
 */
#ifndef MB_TIME_H_
#define MB_TIME_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MB_TIME_OK 0
#define MB_TIME_INVALID_ARG (-1)        /* null pointer, count < 2, non-finite or non-positive time */
#define MB_TIME_BAD_CU_SEQLENS (-2)     /* cu[0] != 0 or decreasing */
#define MB_TIME_NOT_IDENTIFIABLE (-3)   /* the profile does not determine alpha and beta */

typedef struct {
  double alpha; /* time per token (linear part: MLP and everything else that scales with N) */
  double beta;  /* time per squared document length (attention) */
} mb_time_model;

/* N = sum l_i and sum l_i^2 of one packed micro-batch, exact in int64.
 * cu_seqlens: num_docs + 1 entries, cu[0] = 0, non-decreasing (empty documents are legal). */
int mb_time_features(const int32_t* cu_seqlens, int32_t num_docs, int64_t* n_tokens,
                     int64_t* sum_sq);

/* Least-squares fit of Eq. 1 (no intercept) to `count` profiled micro-batches:
 * times[i] ~ alpha * n_tokens[i] + beta * sum_sq[i].  Any time unit; the model keeps it. */
int mb_time_fit(const int64_t* n_tokens, const int64_t* sum_sq, const double* times,
                int32_t count, mb_time_model* model);

/* Eq. 1. */
double mb_time_predict(const mb_time_model* model, int64_t n_tokens, int64_t sum_sq);

/* Mean absolute percentage error of the model over `count` micro-batches (NaN on bad input). */
double mb_time_mape_percent(const mb_time_model* model, const int64_t* n_tokens,
                            const int64_t* sum_sq, const double* times, int32_t count);

/* 1 if observed > predicted * (1 + threshold), else 0; the paper's threshold is 0.25. */
int mb_time_is_suspicious(double observed, double predicted, double threshold);

#ifdef __cplusplus
}
#endif
#endif /* MB_TIME_H_ */
