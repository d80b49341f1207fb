// Micro-batch time predictor of Section 5.2 (Eq. 1) and the 25 % filter: host code.
// The 2 x 2 normal equations are formed from columns scaled to unit root-mean-square (token
// counts are ~1e3..1e5, squared lengths ~1e5..1e9) and solved in long double.
#include "mb_time.h"

#include <cmath>
#include <limits>

namespace {

struct Sums {
  long double aa = 0, ab = 0, bb = 0, at = 0, bt = 0;
};

}  // namespace

extern "C" {

int mb_time_features(const int32_t* cu, int32_t num_docs, int64_t* n_tokens, int64_t* sum_sq) {
  if (!cu || !n_tokens || !sum_sq || num_docs < 1) return MB_TIME_INVALID_ARG;
  if (cu[0] != 0) return MB_TIME_BAD_CU_SEQLENS;
  int64_t n = 0, s = 0;
  for (int32_t b = 0; b < num_docs; ++b) {
    const int64_t l = (int64_t)cu[b + 1] - cu[b];
    if (l < 0) return MB_TIME_BAD_CU_SEQLENS;
    n += l;
    s += l * l;
  }
  *n_tokens = n;
  *sum_sq = s;
  return MB_TIME_OK;
}

int mb_time_fit(const int64_t* n_tokens, const int64_t* sum_sq, const double* times,
                int32_t count, mb_time_model* model) {
  if (!n_tokens || !sum_sq || !times || !model || count < 2) return MB_TIME_INVALID_ARG;
  long double ra = 0, rb = 0;
  for (int32_t i = 0; i < count; ++i) {
    if (!(times[i] > 0) || !std::isfinite(times[i]) || n_tokens[i] < 0 || sum_sq[i] < 0)
      return MB_TIME_INVALID_ARG;
    ra += (long double)n_tokens[i] * n_tokens[i];
    rb += (long double)sum_sq[i] * sum_sq[i];
  }
  if (!(ra > 0) || !(rb > 0)) return MB_TIME_NOT_IDENTIFIABLE;
  const long double sa = std::sqrt(ra / count), sb = std::sqrt(rb / count);
  Sums m;
  for (int32_t i = 0; i < count; ++i) {
    const long double a = n_tokens[i] / sa, b = sum_sq[i] / sb, t = times[i];
    m.aa += a * a; m.ab += a * b; m.bb += b * b; m.at += a * t; m.bt += b * t;
  }
  // scaled columns have squared norm `count` each; det / count^2 = 1 - cos^2 of their angle
  const long double det = m.aa * m.bb - m.ab * m.ab;
  if (!(det > 1e-12L * m.aa * m.bb)) return MB_TIME_NOT_IDENTIFIABLE;
  model->alpha = (double)((m.at * m.bb - m.bt * m.ab) / det / sa);
  model->beta = (double)((m.aa * m.bt - m.ab * m.at) / det / sb);
  return MB_TIME_OK;
}

double mb_time_predict(const mb_time_model* model, int64_t n_tokens, int64_t sum_sq) {
  if (!model) return std::numeric_limits<double>::quiet_NaN();
  return model->alpha * (double)n_tokens + model->beta * (double)sum_sq;
}

double mb_time_mape_percent(const mb_time_model* model, const int64_t* n_tokens,
                            const int64_t* sum_sq, const double* times, int32_t count) {
  if (!model || !n_tokens || !sum_sq || !times || count < 1)
    return std::numeric_limits<double>::quiet_NaN();
  long double acc = 0;
  for (int32_t i = 0; i < count; ++i) {
    if (!(times[i] > 0)) return std::numeric_limits<double>::quiet_NaN();
    acc += std::fabs(mb_time_predict(model, n_tokens[i], sum_sq[i]) - times[i]) / times[i];
  }
  return (double)(acc / count * 100.0L);
}

int mb_time_is_suspicious(double observed, double predicted, double threshold) {
  return observed > predicted * (1.0 + threshold) ? 1 : 0;
}

}  // extern "C"
