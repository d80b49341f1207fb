// Forward kernel and the reduction of its cut chains.
#ifndef VARLEN_ATTN_FWD_HPP_
#define VARLEN_ATTN_FWD_HPP_

#include "tiles.hpp"
#include "staging.hpp"
#include "fragments.hpp"
#include "plan.hpp"

namespace {

// ----------------------------------------------------------------------------------------
// Forward.  One workgroup per (row unit, q head); wave w owns query rows row0 + 32w .. +31.
// Computes S^T = K Q^T so that a query is a lane column; online softmax in the exp2 domain
// with a lazily updated running max; O^T += V^T P^T.  A unit that covers its whole chain
// normalises and stores O and LSE; otherwise it stores the unnormalised accumulator with its
// running max and row sum for fwd_combine_kernel.
// ----------------------------------------------------------------------------------------
template <int D, bool SELF>
__global__ void __launch_bounds__(kThreads, 2)
fwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
           const varlen_attn_plan_header* __restrict__ hdr,
           const varlen_attn_unit* __restrict__ units, __bf16* __restrict__ o,
           float* __restrict__ lse, float* __restrict__ partials, int N, int Hq, int Hkv,
           float scale, int max_units, PlanArgs plan) {
  constexpr int KK = D / 16, DB = D / 32;
  constexpr int NS = 4;                              // pipeline stages of 32 keys
  constexpr int kStageBytes = kSub * D * 2;
  constexpr int LPS = 2 * StageLoader<D>::kPerWave;  // DMA loads per thread per stage (K and V)
  __shared__ __attribute__((aligned(1024))) char smem[2 * NS * kStageBytes];  // K stages, V stages

  int unit_idx, head;
  varlen_attn_unit it;
  if (SELF) {
    // Small microbatch: no plan launch in front.  Workgroup 0 makes the plan (for the reduction
    // of this forward and for the backward) while the others work out their own unit from
    // cu_seqlens, in the order (tile, chunk), by the plan's rules.
    __shared__ varlen_attn_unit own_unit;
    __shared__ int own_valid;
    if (blockIdx.x == 0) {
      if (threadIdx.x < kPlanThreadsSmall) plan_body<kPlanThreadsSmall>(plan);
      return;
    }
    decode_block(blockIdx.x - 1, Hq, unit_idx, head);
    if (threadIdx.x < 64) {
      varlen_attn_unit mine;
      const bool ok = derive_row_unit(plan.cu, plan.B, plan.N, Hq, plan.no_split, plan.force_ch[0],
                                      plan.slots_cap, unit_idx, threadIdx.x, mine);
      if (threadIdx.x == 0) { own_valid = ok ? 1 : 0; if (ok) own_unit = mine; }
    }
    __syncthreads();
    if (!own_valid) return;
    // (scalar registers again: everything derived from the unit stays wave-uniform)
    it = varlen_attn_unit{__builtin_amdgcn_readfirstlane(own_unit.row0), __builtin_amdgcn_readfirstlane(own_unit.doc_start),
                          __builtin_amdgcn_readfirstlane(own_unit.doc_end), __builtin_amdgcn_readfirstlane(own_unit.step_begin),
                          __builtin_amdgcn_readfirstlane(own_unit.step_end), __builtin_amdgcn_readfirstlane(own_unit.slot),
                          __builtin_amdgcn_readfirstlane(own_unit.cost), 0};
  } else {
    decode_block(blockIdx.x, Hq, unit_idx, head);
    // both loads in flight together; the unit array always has max_units >= grid / Hq entries
    const int n_units = hdr->n_row_units;
    it = units[min(unit_idx, max_units - 1)];
    if (unit_idx >= n_units) return;
  }
  const int kvh = head / (Hq / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, c = lane & 31;
  const float cs = scale * kLog2e;

  const int wave_row0 = it.row0 + 32 * wave;
  const int my_row = wave_row0 + c;
  const bool row_valid = my_row < it.doc_end;
  const bool wave_active = wave_row0 < it.doc_end;
  const int wave_last_row = min(wave_row0 + 31, it.doc_end - 1);
  const int wg_last_row = min(it.row0 + kTile, it.doc_end) - 1;
  const int kv_begin = it.doc_start + it.step_begin * kStep;
  const int kv_end = min(it.doc_start + it.step_end * kStep, wg_last_row + 1);
  const int n_sub = (kv_end - kv_begin + kSub - 1) / kSub;

  const __bf16* kbase = k + (size_t)kvh * D;
  const __bf16* vbase = v + (size_t)kvh * D;
  const size_t kv_stride = (size_t)Hkv * D;
  const unsigned lds_k = lds_addr_of(smem), lds_v = lds_k + NS * kStageBytes;

  StageLoader<D> loader;
  loader.init(wave, lane, (unsigned)(kv_stride * 2));
  // stages are issued in order, one call per sub-step: the wave-uniform addresses of the next
  // stage's first K and V rows live in scalar registers and move on by one stage per call
  const unsigned long long kStageStride = (unsigned long long)kSub * (kv_stride * 2);
  unsigned long long k_next = uniform64(reinterpret_cast<const char*>(kbase) + (size_t)kv_begin * (kv_stride * 2));
  unsigned long long v_next = uniform64(reinterpret_cast<const char*>(vbase) + (size_t)kv_begin * (kv_stride * 2));
  auto issue = [&](int sub, int stage) {
    const int row0 = kv_begin + kSub * min(sub, n_sub - 1);
    loader.issue_at(k_next, row0, it.doc_end - 1, lds_k + stage * kStageBytes, wave);
    loader.issue_at(v_next, row0, it.doc_end - 1, lds_v + stage * kStageBytes, wave);
    if (sub < n_sub - 1) { k_next += kStageStride; v_next += kStageStride; }
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st) issue(st, st);

  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 t = {0, 0, 0, 0};
    if (row_valid)
      t = *reinterpret_cast<const uint4*>(q + ((size_t)my_row * Hq + head) * D + 16 * kk + 8 * h);
    qf[kk] = __builtin_bit_cast(bf16x8, t);
  }
  FragOffsets<D> fo;
  fo.init(lane);
  // Let the compiler see its own loads complete here, once; otherwise it keeps a vmcnt(0)
  // for them inside the loop, which would also wait for every prefetch in flight.
  wait_all_vm_visible();

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) oacc[i] = f32x16(0.f);
  float m_run = -INFINITY, l_run = 0.f;

  // one sub-step: 32 keys against this wave's 32 queries, stage index known at compile time
  auto compute = [&](int sub, auto stage_c) {
    constexpr int ST = decltype(stage_c)::value;
    const int kv0 = kv_begin + kSub * sub;
    if (!(wave_active && kv0 <= wave_last_row)) return;
    const char* kt = smem + ST * kStageBytes;
    const char* vt = smem + (NS + ST) * kStageBytes;
    f32x16 s = f32x16(0.f);
    __builtin_amdgcn_s_setprio(2);   // matrix phases win the issue slot over the other wave's softmax
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) s = mfma(lds_read_frag(kt, fo.row_frag[kk]), qf[kk], s);
    __builtin_amdgcn_s_setprio(0);
    // the transposed V fragments of the second contraction are requested before the softmax
    // arithmetic, so that they arrive behind it
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 vtf[2][DB];
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
      for (int db = 0; db < DB; ++db) vtf[cc][db] = read_trans<D>(vt, fo, cc, db);
    __builtin_amdgcn_sched_barrier(0);
    if (kv0 + kSub - 1 > wave_row0) {  // touches the diagonal for some row
      const int t = my_row - kv0 - 4 * h;  // key offset 8 (r / 4) + r % 4 is allowed iff <= t
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (8 * (r / 4) + (r % 4) > t) s[r] = -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = __builtin_fmaxf(mx, s[r]);
    mx = half_max(mx);
    const float m_new = __builtin_fmaxf(m_run, mx * cs);
    if (__any(m_new > m_run + kRescaleTau)) {
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] *= alpha;
    }
    float psum = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cs, -m_run));
      s[r] = p;
      psum += p;
    }
    l_run += psum;
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const bf16x8 pb = pack8(s, 8 * cc);
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma(vtf[cc][db], pb, oacc[db]);
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // iteration `sub`: its stage has landed once at most NS-2 newer stages are in flight; the
  // barrier also tells that every wave is done with the stage about to be refilled
  auto body = [&](int sub, auto stage_c) {
    constexpr int ST = decltype(stage_c)::value;
    wait_vm<(NS - 2) * LPS>();
    __syncthreads();
    issue(sub + NS - 1, (ST + NS - 1) % NS);
    compute(sub, stage_c);
  };
  for (int sub = 0; sub < n_sub; sub += NS) {
    body(sub, std::integral_constant<int, 0>{});
    if (sub + 1 >= n_sub) break;
    body(sub + 1, std::integral_constant<int, 1>{});
    if (sub + 2 >= n_sub) break;
    body(sub + 2, std::integral_constant<int, 2>{});
    if (sub + 3 >= n_sub) break;
    body(sub + 3, std::integral_constant<int, 3>{});
  }
  wait_vm<0>();  // nothing may still be landing in LDS when the workgroup retires

  if (it.slot >= 0) {
    // a wave that saw no key in this chunk leaves the neutral element (0, -inf, 0)
    float* part = partials + ((size_t)it.slot * Hq + head) * fwd_partial_floats<D>();
    store_frag<D>(part, oacc, wave, lane);
    part[frag_floats<D>() + tid] = m_run;
    part[frag_floats<D>() + kThreads + tid] = l_run;
    return;
  }
  if (!wave_active) return;
  const float l_tot = half_sum(l_run);
  if (row_valid) {
    store_rows<D>(o + ((size_t)my_row * Hq + head) * D, oacc, h, 1.0f / l_tot);
    if (h == 0) lse[(size_t)head * N + my_row] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}

// Sums the chunks of a cut row chain:  O = sum_c 2^(m_c - m) O_c / sum_c 2^(m_c - m) l_c.
// Elementwise over the fragment layout: thread t of an (item, head) owns float4 number t of
// every partial (so all loads are contiguous), chunks are taken in chain order.
template <int D>
__global__ void __launch_bounds__(kThreads)
fwd_combine_kernel(const varlen_attn_plan_header* __restrict__ hdr,
                   const varlen_attn_combine_item* __restrict__ items,
                   const float* __restrict__ partials, __bf16* __restrict__ o,
                   float* __restrict__ lse, int N, int Hq) {
  constexpr int DB = D / 32;
  constexpr int kBlocksPerItem = kTile * D / 4 / kThreads;
  const int sub = blockIdx.x % kBlocksPerItem, rest = blockIdx.x / kBlocksPerItem;
  const int idx = rest / Hq, head = rest % Hq;
  if (idx >= hdr->n_row_combine) return;
  const varlen_attn_combine_item it = items[idx];
  const int t = sub * kThreads + threadIdx.x;  // float4 index inside the fragment
  const int lane = t & 63, rq = (t >> 6) & 3, db = (t >> 8) % DB, wave = (t >> 8) / DB;
  const int h = lane >> 5, c = lane & 31;
  const int my_row = it.row0 + 32 * wave + c;
  if (my_row >= it.doc_end) return;
  const size_t pstride = (size_t)Hq * fwd_partial_floats<D>();
  const float* p0 = partials + ((size_t)it.slot0 * Hq + head) * fwd_partial_floats<D>();
  const float* st = p0 + frag_floats<D>() + wave * 64;  // m[lane], then l[lane] 256 floats on
  float m = -INFINITY;
  for (int ch = 0; ch < it.n_chunks; ++ch) m = __builtin_fmaxf(m, st[ch * pstride + lane]);
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int ch = 0; ch < it.n_chunks; ++ch) {
    const float w = __builtin_amdgcn_exp2f(st[ch * pstride + lane] - m);
    l += w * (st[ch * pstride + kThreads + c] + st[ch * pstride + kThreads + 32 + c]);
    const f32x4 x = *reinterpret_cast<const f32x4*>(p0 + ch * pstride + (size_t)t * 4);
    acc += w * x;
  }
  const float inv = 1.0f / l;
  *reinterpret_cast<uint2*>(o + ((size_t)my_row * Hq + head) * D + 32 * db + 8 * rq + 4 * h) =
      pack4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
  if (db == 0 && rq == 0 && h == 0)
    lse[(size_t)head * N + my_row] = (m + __builtin_amdgcn_logf(l)) * kLn2;
}

}  // namespace

#endif  // VARLEN_ATTN_FWD_HPP_
