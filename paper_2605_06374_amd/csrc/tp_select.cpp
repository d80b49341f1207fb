// TP subgroup selection of Section 6.1 (Eq. 3 and Eq. 4): host code.
// One stable sort of the surviving devices by throughput; the minimum of the top-k prefix is
// then the k-th entry, so every feasible degree costs one multiplication.
#include "tp_select.h"

#include <algorithm>
#include <cmath>

extern "C" int tp_select_subgroup(const double* p, const uint8_t* fail_stop, int32_t n,
                                  int32_t k_min, int32_t* degree, double* aggregate,
                                  int32_t* role) {
  if (!p || !fail_stop || !degree || !aggregate || !role || n < 1 || n > 64 || k_min < 1)
    return TP_SELECT_INVALID_ARG;
  int ranked[64];
  int alive = 0;
  for (int i = 0; i < n; ++i) {
    if (fail_stop[i]) continue;
    if (!(p[i] >= 0) || !std::isfinite(p[i])) return TP_SELECT_INVALID_ARG;
    ranked[alive++] = i;
  }
  std::stable_sort(ranked, ranked + alive, [&](int a, int b) { return p[a] > p[b]; });
  int best_k = 0;
  double best = 0.0;
  for (int k = 1; k <= alive; k *= 2) {
    if (k < k_min) continue;
    const double value = k * p[ranked[k - 1]];
    if (best_k == 0 || value >= best) { best_k = k; best = value; }   // ties: larger degree
  }
  for (int i = 0; i < n; ++i) role[i] = fail_stop[i] ? TP_SELECT_ROLE_FAIL_STOP : TP_SELECT_ROLE_STANDBY;
  for (int r = 0; r < best_k; ++r) role[ranked[r]] = TP_SELECT_ROLE_MEMBER;
  *degree = best_k;
  *aggregate = best;
  return best_k ? TP_SELECT_OK : TP_SELECT_NO_FEASIBLE_DEGREE;
}
