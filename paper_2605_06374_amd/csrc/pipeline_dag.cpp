// Iteration-time predictor of Section 5.2 (Eq. 2): host code.
// The DAG is never materialised as edge lists: every vertex has at most three predecessors
// that follow from its kind and its position in its stage's order, so the start times are
// relaxed stage by stage with one cursor per stage until every cursor reaches the end of its
// list (a sweep in which no cursor moves means the order contradicts the data dependencies).
#include "pipeline_dag.h"

#include <algorithm>
#include <vector>

namespace {

inline size_t at(int kind, int m, int s, int M, int S) { return ((size_t)kind * M + m) * S + s; }

}  // namespace

extern "C" {

int pipeline_dag_schedule_1f1b(int32_t S, int32_t M, pipeline_dag_chunk* order) {
  if (S < 1 || M < 1 || !order) return PIPELINE_DAG_INVALID_ARG;
  for (int s = 0; s < S; ++s) {
    pipeline_dag_chunk* o = order + (size_t)s * 2 * M;
    const int warm = std::min(S - 1 - s, M);
    int n = 0;
    for (int m = 0; m < warm; ++m) o[n++] = {PIPELINE_DAG_F, m};
    for (int i = 0; i + warm < M; ++i) {
      o[n++] = {PIPELINE_DAG_F, warm + i};
      o[n++] = {PIPELINE_DAG_B, i};
    }
    for (int i = M - warm; i < M; ++i) o[n++] = {PIPELINE_DAG_B, i};
  }
  return PIPELINE_DAG_OK;
}

int pipeline_dag_schedule_zbh1(int32_t S, int32_t M, pipeline_dag_chunk* order) {
  if (S < 1 || M < 1 || !order) return PIPELINE_DAG_INVALID_ARG;
  constexpr int kNever = 1 << 30;
  // finish step of F and B chunks under unit costs
  std::vector<int> f_done((size_t)M * S, kNever), b_done((size_t)M * S, kNever);
  std::vector<int> nf(S, 0), nb(S, 0), nw(S, 0), len(S, 0);
  struct Pick { int stage, kind, m; };
  std::vector<Pick> picks;
  const long long limit = 16LL * (M + S) + 16;
  for (long long t = 0;; ++t) {
    bool all = true;
    for (int s = 0; s < S; ++s) all = all && nw[s] == M;
    if (all) break;
    if (t > limit) return PIPELINE_DAG_BAD_SCHEDULE;   // cannot happen for S, M >= 1
    picks.clear();
    for (int s = 0; s < S; ++s) {
      if (nb[s] < M) {
        const int m = nb[s];
        const int dep = s + 1 < S ? b_done[(size_t)m * S + s + 1] : f_done[(size_t)m * S + s];
        if (dep <= t && f_done[(size_t)m * S + s] <= t) { picks.push_back({s, PIPELINE_DAG_B, m}); continue; }
      }
      if (nf[s] < M && nf[s] - nb[s] < S - s) {
        const int m = nf[s];
        if (s == 0 || f_done[(size_t)m * S + s - 1] <= t) { picks.push_back({s, PIPELINE_DAG_F, m}); continue; }
      }
      if (nw[s] < nb[s]) picks.push_back({s, PIPELINE_DAG_W, nw[s]});
    }
    for (const Pick& p : picks) {
      order[(size_t)p.stage * 3 * M + len[p.stage]++] = {p.kind, p.m};
      if (p.kind == PIPELINE_DAG_F) { f_done[(size_t)p.m * S + p.stage] = (int)t + 1; ++nf[p.stage]; }
      else if (p.kind == PIPELINE_DAG_B) { b_done[(size_t)p.m * S + p.stage] = (int)t + 1; ++nb[p.stage]; }
      else ++nw[p.stage];
    }
  }
  return PIPELINE_DAG_OK;
}

int pipeline_dag_simulate(int32_t S, int32_t M, int32_t kinds, const pipeline_dag_chunk* order,
                          const double* cost, double p2p, double* iteration_time,
                          double* t_start_out) {
  if (S < 1 || M < 1 || (kinds != 2 && kinds != 3) || !order || !cost || !iteration_time ||
      !(p2p >= 0))
    return PIPELINE_DAG_INVALID_ARG;
  const int per_stage = kinds * M;
  const size_t nv = (size_t)kinds * M * S;
  for (size_t i = 0; i < nv; ++i)
    if (!(cost[i] >= 0)) return PIPELINE_DAG_INVALID_ARG;
  // every chunk of a stage exactly once
  std::vector<char> seen(nv, 0);
  for (int s = 0; s < S; ++s)
    for (int p = 0; p < per_stage; ++p) {
      const pipeline_dag_chunk c = order[(size_t)s * per_stage + p];
      if (c.kind < 0 || c.kind >= kinds || c.microbatch < 0 || c.microbatch >= M)
        return PIPELINE_DAG_INVALID_ARG;
      char& f = seen[at(c.kind, c.microbatch, s, M, S)];
      if (f) return PIPELINE_DAG_BAD_SCHEDULE;
      f = 1;
    }
  std::vector<double> start(nv, 0.0);
  std::vector<char> done(nv, 0);
  std::vector<int> cur(S, 0);
  std::vector<double> stage_free(S, 0.0);   // completion of the previous chunk of the stage
  size_t left = nv;
  while (left) {
    bool moved = false;
    for (int s = 0; s < S; ++s) {
      while (cur[s] < per_stage) {
        const pipeline_dag_chunk c = order[(size_t)s * per_stage + cur[s]];
        const int m = c.microbatch;
        double t = stage_free[s];
        bool ready = true;
        auto need = [&](int kind, int stage, double edge) {
          const size_t u = at(kind, m, stage, M, S);
          if (!done[u]) { ready = false; return; }
          t = std::max(t, start[u] + cost[u] + edge);
        };
        if (c.kind == PIPELINE_DAG_F) {
          if (s > 0) need(PIPELINE_DAG_F, s - 1, p2p);
        } else if (c.kind == PIPELINE_DAG_B) {
          need(PIPELINE_DAG_F, s, 0.0);
          if (s + 1 < S) need(PIPELINE_DAG_B, s + 1, p2p);
        } else {
          need(PIPELINE_DAG_B, s, 0.0);
        }
        if (!ready) break;
        const size_t v = at(c.kind, m, s, M, S);
        start[v] = t;
        done[v] = 1;
        stage_free[s] = t + cost[v];
        ++cur[s];
        --left;
        moved = true;
      }
    }
    if (!moved) return PIPELINE_DAG_BAD_SCHEDULE;
  }
  double total = 0.0;
  for (int s = 0; s < S; ++s) total = std::max(total, stage_free[s]);
  *iteration_time = total;
  if (t_start_out) std::copy(start.begin(), start.end(), t_start_out);
  return PIPELINE_DAG_OK;
}

}  // extern "C"
