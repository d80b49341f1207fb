// Backward kernels (dQ; dK and dV) and the reduction of their partial results.
#ifndef VARLEN_ATTN_BWD_HPP_
#define VARLEN_ATTN_BWD_HPP_

#include "tiles.hpp"
#include "staging.hpp"
#include "fragments.hpp"

namespace {

// ----------------------------------------------------------------------------------------
// Backward, dQ (first backward kernel).  Same decomposition as the forward: one workgroup per
// (row unit, q head).  Its prologue also computes D = rowsum(dO * O) for its rows.
// S^T = K Q^T, dP^T = V dO^T, dS^T = P^T (dP^T - D), dQ^T += K^T dS^T.
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads, 2)
bwd_dq_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
              const __bf16* __restrict__ v, const __bf16* __restrict__ o,
              const __bf16* __restrict__ d_o, const float* __restrict__ lse,
              float* __restrict__ dsum, float* __restrict__ lse2_out,
              const varlen_attn_plan_header* __restrict__ hdr,
              const varlen_attn_unit* __restrict__ units, __bf16* __restrict__ dq,
              float* __restrict__ partials, int N, int Hq, int Hkv, float scale,
              int max_units) {
  constexpr int KK = D / 16, DB = D / 32;
  constexpr int NS = 4;
  constexpr int kStageBytes = kSub * D * 2;
  constexpr int LPS = 2 * StageLoader<D>::kPerWave;
  __shared__ __attribute__((aligned(1024))) char smem[2 * NS * kStageBytes];  // K stages, V stages

  int unit_idx, head;
  decode_block(blockIdx.x, Hq, unit_idx, head);
  // both loads in flight together; the unit array always has max_units >= grid / Hq entries
  const int n_units = hdr->n_row_units;
  const varlen_attn_unit it = units[min(unit_idx, max_units - 1)];
  if (unit_idx >= n_units) return;
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
  const unsigned lds_k = lds_addr_of(smem), lds_v = lds_k + NS * kStageBytes;

  StageLoader<D> loader;
  loader.init(wave, lane, (unsigned)((size_t)Hkv * D * 2));
  // stages are issued in order, one call per sub-step: the wave-uniform addresses of the next
  // stage's first K and V rows live in scalar registers and move on by one stage per call
  const unsigned long long kStageStride = (unsigned long long)kSub * ((size_t)Hkv * D * 2);
  unsigned long long k_next = uniform64(reinterpret_cast<const char*>(kbase) + (size_t)kv_begin * ((size_t)Hkv * D * 2));
  unsigned long long v_next = uniform64(reinterpret_cast<const char*>(vbase) + (size_t)kv_begin * ((size_t)Hkv * D * 2));
  auto issue = [&](int sub, int stage) {
    const int row0 = kv_begin + kSub * min(sub, n_sub - 1);
    loader.issue_at(k_next, row0, it.doc_end - 1, lds_k + stage * kStageBytes, wave);
    loader.issue_at(v_next, row0, it.doc_end - 1, lds_v + stage * kStageBytes, wave);
    if (sub < n_sub - 1) { k_next += kStageStride; v_next += kStageStride; }
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st) issue(st, st);

  // Q and dO fragments stay in registers; the O fragments are only needed for
  // D = rowsum(dO * O): each lane holds half of its row's columns, the other half-wave the rest.
  bf16x8 qf[KK], dof[KK];
  float d_part = 0.f;
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 t = {0, 0, 0, 0}, u = {0, 0, 0, 0}, w = {0, 0, 0, 0};
    if (row_valid) {
      const size_t off = ((size_t)my_row * Hq + head) * D + 16 * kk + 8 * h;
      t = *reinterpret_cast<const uint4*>(q + off);
      u = *reinterpret_cast<const uint4*>(d_o + off);
      w = *reinterpret_cast<const uint4*>(o + off);
    }
    qf[kk] = __builtin_bit_cast(bf16x8, t);
    dof[kk] = __builtin_bit_cast(bf16x8, u);
    const bf16x8 of = __builtin_bit_cast(bf16x8, w);
#pragma unroll
    for (int e = 0; e < 8; ++e) d_part += (float)dof[kk][e] * (float)of[e];
  }
  const float dsum_row = half_sum(d_part);
  // rows past the document end get LSE = +huge so that their P is exactly 0
  const float lse2 = row_valid ? lse[(size_t)head * N + my_row] * kLog2e : 1e30f;
  // the unit that starts the chain publishes D and LSE * log2(e) for the dK/dV kernel
  if (it.step_begin == 0 && row_valid && h == 0) {
    dsum[(size_t)head * N + my_row] = dsum_row;
    lse2_out[(size_t)head * N + my_row] = lse2;
  }
  FragOffsets<D> fo;
  fo.init(lane);
  wait_all_vm_visible();

  f32x16 acc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) acc[i] = f32x16(0.f);

  auto compute = [&](int sub, auto stage_c) {
    constexpr int ST = decltype(stage_c)::value;
    const int kv0 = kv_begin + kSub * sub;
    if (!(wave_active && kv0 <= wave_last_row)) return;
    const char* kt = smem + ST * kStageBytes;
    const char* vt = smem + (NS + ST) * kStageBytes;
    f32x16 s = f32x16(0.f), dp = f32x16(0.f);
    __builtin_amdgcn_s_setprio(2);   // matrix phases win the issue slot over the other wave's vector work
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      s = mfma(lds_read_frag(kt, fo.row_frag[kk]), qf[kk], s);
      dp = mfma(lds_read_frag(vt, fo.row_frag[kk]), dof[kk], dp);
    }
    __builtin_amdgcn_s_setprio(0);
    // the transposed K fragments of the last contraction are requested before the vector
    // work, so that they arrive behind it
    __builtin_amdgcn_sched_barrier(0);
    bf16x8 ktf[2][DB];
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
      for (int db = 0; db < DB; ++db) ktf[cc][db] = read_trans<D>(kt, fo, cc, db);
    __builtin_amdgcn_sched_barrier(0);
    if (kv0 + kSub - 1 > wave_row0) {  // touches the diagonal for some row (wave-uniform)
      const int t = my_row - kv0 - 4 * h;  // key offset 8 (r / 4) + r % 4 is allowed iff <= t
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cs, -lse2));
        if (8 * (r / 4) + (r % 4) > t) p = 0.f;
        s[r] = p * (dp[r] - dsum_row);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cs, -lse2));
        s[r] = p * (dp[r] - dsum_row);
      }
    }
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const bf16x8 dsb = pack8(s, 8 * cc);
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(ktf[cc][db], dsb, acc[db]);
    }
    __builtin_amdgcn_s_setprio(0);
  };
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
    store_frag<D>(partials + ((size_t)it.slot * Hq + head) * frag_floats<D>(), acc, wave, lane);
    return;
  }
  if (row_valid) store_rows<D>(dq + ((size_t)my_row * Hq + head) * D, acc, h, scale);
}

// ----------------------------------------------------------------------------------------
// Fused backward (VARLEN_ATTN_FLAG_FUSED_BWD), first kernel: D = rowsum(dO * O) and
// LSE * log2(e) for every (token, q head) into the workspace, and the fp32 dQ accumulator
// cleared.  One group of D / 8 lanes per row (16 bytes per lane); HBM-bound.
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads)
bwd_prep_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ d_o,
                const float* __restrict__ lse, float* __restrict__ dsum,
                float* __restrict__ lse2_out, float* __restrict__ dq_acc, int N, int Hq) {
  constexpr int kLanesPerRow = D / 8;
  constexpr int kRowsPerBlock = kThreads / kLanesPerRow;
  const long long row = (long long)blockIdx.x * kRowsPerBlock + threadIdx.x / kLanesPerRow;  // t * Hq + h
  const int part = threadIdx.x % kLanesPerRow;
  const bool valid = row < (long long)N * Hq;
  float acc = 0.f;
  if (valid) {
    const uint4 a = *reinterpret_cast<const uint4*>(d_o + row * D + 8 * part);
    const uint4 b = *reinterpret_cast<const uint4*>(o + row * D + 8 * part);
    const bf16x8 x = __builtin_bit_cast(bf16x8, a), y = __builtin_bit_cast(bf16x8, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)x[e] * (float)y[e];
    f32x4* z = reinterpret_cast<f32x4*>(dq_acc + row * D + 8 * part);
    z[0] = f32x4{0.f, 0.f, 0.f, 0.f};
    z[1] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int off = kLanesPerRow / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if (part == 0 && valid) {
    const int t = (int)(row / Hq), h = (int)(row % Hq);
    dsum[(size_t)h * N + t] = acc;
    lse2_out[(size_t)h * N + t] = lse[(size_t)h * N + t] * kLog2e;
  }
}

// Fused backward, last kernel: dQ = scale * accumulator, rounded to bf16.
template <int D>
__global__ void __launch_bounds__(kThreads)
bwd_dq_finish_kernel(const float* __restrict__ dq_acc, __bf16* __restrict__ dq, long long n8,
                     float scale) {
  const long long i = (long long)blockIdx.x * kThreads + threadIdx.x;   // group of 8 elements
  if (i >= n8) return;
  const f32x4 a = reinterpret_cast<const f32x4*>(dq_acc)[2 * i], b = reinterpret_cast<const f32x4*>(dq_acc)[2 * i + 1];
  const uint2 lo = pack4(a[0] * scale, a[1] * scale, a[2] * scale, a[3] * scale);
  const uint2 hi = pack4(b[0] * scale, b[1] * scale, b[2] * scale, b[3] * scale);
  reinterpret_cast<uint4*>(dq)[i] = uint4{lo.x, lo.y, hi.x, hi.y};
}

// Sum of the dQ partials of one cut tile and q head by one whole workgroup (thread t owns the
// float4s t, t + 256, ... of the fragment; chunks are added in chain order, as many loads in
// flight as four chunks of four float4s).  These workgroups ride at the end of the dK/dV
// kernel's grid: the dQ partials are complete when that kernel starts, and its last round
// leaves most compute units idle, so the reduction costs no launch and no time of its own.
template <int D>
__device__ __forceinline__ void dq_tile_combine(int block, const varlen_attn_plan_header* __restrict__ hdr,
                                                int max_items,
                                                const varlen_attn_combine_item* __restrict__ items,
                                                const float* __restrict__ partials,
                                                __bf16* __restrict__ dq, int Hq, float scale) {
  constexpr int DB = D / 32;
  constexpr int kPerThread = kTile * D / 4 / kThreads;   // float4s of a fragment per thread
  const int idx = block / Hq, head = block % Hq;
  // both loads in flight together
  const int n_items = hdr->n_row_combine;
  const varlen_attn_combine_item it = items[min(idx, max_items - 1)];
  if (idx >= n_items) return;
  const size_t pstride = (size_t)Hq * frag_floats<D>();
  const float* p0 = partials + ((size_t)it.slot0 * Hq + head) * frag_floats<D>() + (size_t)threadIdx.x * 4;
#pragma unroll 1
  for (int s0 = 0; s0 < kPerThread; s0 += 4) {
    f32x4 acc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
    for (int c0 = 0; c0 < it.n_chunks; c0 += 4) {
      f32x4 x[4][4];
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          x[j][u] = f32x4{0.f, 0.f, 0.f, 0.f};
          if (c0 + j < it.n_chunks)   // the same for the whole workgroup
            x[j][u] = *reinterpret_cast<const f32x4*>(p0 + (size_t)(c0 + j) * pstride +
                                                      (size_t)(s0 + u) * kThreads * 4);
        }
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (c0 + j < it.n_chunks) acc[u] += x[j][u];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = (s0 + u) * kThreads + threadIdx.x;
      const int lane = t & 63, rq = (t >> 6) & 3, db = (t >> 8) % DB, wave = (t >> 8) / DB;
      const int h = lane >> 5, c = lane & 31;
      const int my_row = it.row0 + 32 * wave + c;
      if (my_row < it.doc_end)
        *reinterpret_cast<uint2*>(dq + ((size_t)my_row * Hq + head) * D + 32 * db + 8 * rq + 4 * h) =
            pack4(acc[u][0] * scale, acc[u][1] * scale, acc[u][2] * scale, acc[u][3] * scale);
    }
  }
}

// ----------------------------------------------------------------------------------------
// Backward, dK and dV.  One workgroup per (column unit, q head): wave w owns key rows
// row0 + 32w .. +31, keeps their K and V fragments in registers, and sweeps the unit's
// query steps (from the diagonal towards the document end).
//   S = Q K^T, dP = dO V^T (query rows in registers r, key on the lane),
//   dV^T += dO^T P,  dK^T += Q^T dS.
// With grouped-query attention, or when the chain is cut, the unit stores fp32 partials
// [dK | dV] that bwd_combine_kernel adds up over the chunks and the q heads of the group.
//
// FUSED (VARLEN_ATTN_FLAG_FUSED_BWD): the kernel also forms dQ, so that S and dP are computed
// once for the whole backward (5 contractions instead of 7).  dS of a stage goes, as bf16, into
// an LDS tile [128 keys][64 queries]; one stage later wave w multiplies it with columns
// 32w .. 32w+31 of the unit's K tile (kept in LDS for this) and adds the 64 x 32 block of
// dQ = dS K into a fp32 accumulator in the workspace with floating-point atomics: the order of
// those additions is not fixed, so dQ is not bit-reproducible in this mode.
// ----------------------------------------------------------------------------------------
template <int D, bool FUSED>
__global__ void __launch_bounds__(kThreads, 1)
bwd_dkv_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
               const __bf16* __restrict__ v, const __bf16* __restrict__ d_o,
               const float* __restrict__ lse2, const float* __restrict__ dsum,
               const varlen_attn_plan_header* __restrict__ hdr,
               const varlen_attn_unit* __restrict__ units, __bf16* __restrict__ dk,
               __bf16* __restrict__ dv, float* __restrict__ partials, int N, int Hq, int Hkv,
               float scale, int max_units, int unit_blocks,
               const varlen_attn_combine_item* __restrict__ row_items, int max_items,
               const float* __restrict__ row_partials, __bf16* __restrict__ dq,
               float* __restrict__ dq_acc) {
  constexpr int KK = D / 16, DB = D / 32;
  // Two stages of kStep = 64 query rows: one stage of lookahead is a whole stage of compute
  // (this kernel runs one workgroup per CU), and 64 KB of tiles keeps every LDS offset inside
  // the 16-bit immediate of the read instructions.
  constexpr int NS = 2;
  constexpr int kStageBytes = kStep * D * 2;
  constexpr int kStatBytes = 512;             // lse2[64] then dsum[64], one copy per wave
  using Loader = StageLoader<D, kStep>;
  constexpr int LPS = 2 * Loader::kPerWave + 2;
  constexpr int kPlainBytes = 2 * NS * kStageBytes + NS * 4 * kStatBytes;
  constexpr int kKeyTileBytes = FUSED ? kTile * D * 2 : 0;      // the unit's K rows [128][D]
  constexpr int kDsBytes = FUSED ? kTile * kStep * 2 : 0;       // dS of a stage [128 keys][64 queries]
  // Q stages | dO stages | per-wave stat copies | (fused: K tile | two dS tiles)
  __shared__ __attribute__((aligned(1024))) char smem[kPlainBytes + kKeyTileBytes + 2 * kDsBytes];
  char* const key_tile = smem + kPlainBytes;
  char* const ds_tiles = key_tile + kKeyTileBytes;

  // the workgroups behind the units sum the dQ partials that the dQ kernel left
  if (!FUSED && (int)blockIdx.x >= unit_blocks) {
    dq_tile_combine<D>(blockIdx.x - unit_blocks, hdr, max_items, row_items, row_partials, dq, Hq, scale);
    return;
  }
  int unit_idx, head;
  decode_block(blockIdx.x, Hq, unit_idx, head);
  // both loads in flight together; the unit array always has max_units >= grid / Hq entries
  const int n_units = hdr->n_col_units;
  varlen_attn_unit it = units[min(unit_idx, max_units - 1)];
  // Grouped-query attention on large microbatches: a unit sweeps `hpu` q heads of its group
  // one after the other (dK, dV add up in the registers).  The workgroup ids are then decoded
  // for Hq / hpu head groups, so that the working ones still spread over all XCDs, and the
  // unit is fetched again (one more round trip in front of a long unit).
  const int hpu = hdr->col_heads_per_unit;
  if (hpu > 1) {
    decode_block(blockIdx.x, Hq / hpu, unit_idx, head);
    head *= hpu;
    it = units[min(unit_idx, max_units - 1)];
  }
  if (unit_idx >= n_units) return;
  const int kvh = head / (Hq / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, c = lane & 31;
  const float cs = scale * kLog2e;

  const int wave_kv0 = it.row0 + 32 * wave;
  const int my_kv = wave_kv0 + c;
  const bool kv_valid = my_kv < it.doc_end;
  const bool wave_active = wave_kv0 < it.doc_end;
  const int n_steps = it.step_end - it.step_begin;

  const __bf16* qbase = q + (size_t)head * D;
  const __bf16* dobase = d_o + (size_t)head * D;
  const float* lse_h = lse2 + (size_t)head * N;
  const float* dsum_h = dsum + (size_t)head * N;
  float* dq_acc_h = FUSED ? dq_acc + (size_t)head * D : nullptr;
  int heads_left = hpu;
  const unsigned lds_q = lds_addr_of(smem), lds_do = lds_q + NS * kStageBytes;
  const unsigned lds_stat = lds_do + NS * kStageBytes + wave * kStatBytes;
  const char* stat_base = smem + 2 * NS * kStageBytes + wave * kStatBytes;

  Loader loader;
  loader.init(wave, lane, (unsigned)((size_t)Hq * D * 2));
  // stages are issued in order, one call per step: the wave-uniform addresses of the next
  // stage's first Q and dO rows live in scalar registers and move on by one stage per call
  const unsigned long long kStageStride = (unsigned long long)kStep * ((size_t)Hq * D * 2);
  unsigned long long q_next = 0, do_next = 0;
  auto restart = [&]() {   // at the first step of a chain (of every head the unit sweeps)
    const size_t first = (size_t)(it.row0 + kStep * it.step_begin) * ((size_t)Hq * D * 2);
    q_next = uniform64(reinterpret_cast<const char*>(qbase) + first);
    do_next = uniform64(reinterpret_cast<const char*>(dobase) + first);
  };
  auto issue = [&](int st, int stage) {
    const int q0 = it.row0 + kStep * (it.step_begin + min(st, n_steps - 1));
    loader.issue_at(q_next, q0, it.doc_end - 1, lds_q + stage * kStageBytes, wave);
    loader.issue_at(do_next, q0, it.doc_end - 1, lds_do + stage * kStageBytes, wave);
    dma_floats64(lse_h, q0, it.doc_end - 1, lds_stat + stage * 4 * kStatBytes, lane);
    dma_floats64(dsum_h, q0, it.doc_end - 1, lds_stat + stage * 4 * kStatBytes + 256, lane);
    if (st < n_steps - 1) { q_next += kStageStride; do_next += kStageStride; }
  };
  bf16x8 kf[KK], vf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 t = {0, 0, 0, 0}, u = {0, 0, 0, 0};
    if (kv_valid) {
      const size_t off = ((size_t)my_kv * Hkv + kvh) * D + 16 * kk + 8 * h;
      t = *reinterpret_cast<const uint4*>(k + off);
      u = *reinterpret_cast<const uint4*>(v + off);
    }
    kf[kk] = __builtin_bit_cast(bf16x8, t);
    vf[kk] = __builtin_bit_cast(bf16x8, u);
  }
  FragOffsets<D> fo;
  fo.init(lane);
  if (FUSED) {
    StageLoader<D, kTile> key_loader;
    key_loader.init(wave, lane, (unsigned)((size_t)Hkv * D * 2));
    key_loader.issue(k + (size_t)kvh * D, it.row0, it.doc_end - 1, lds_addr_of(key_tile), wave);
  }
  wait_all_vm_visible();
  // this lane's row of the dS tiles: key 32 wave + c; element (key, query) sits in the 16-byte
  // chunk query / 8 of that row, swizzled like every tile
  // dS of one 32-query block, accumulator registers 8 cc .. 8 cc + 7 (queries 32 qb + 16 cc +
  // 4h + {0..3} and + 8), into the dS tile
  auto ds_store = [&](char* tile, const bf16x8& v, int qb, int cc) __attribute__((always_inline)) {
    const uint4 w = __builtin_bit_cast(uint4, v);
    const int ds_row_swz = swz<kStep>(32 * wave + c);     // recomputed: nothing extra stays live across a stage
    char* row = tile + (32 * wave + c) * (kStep * 2) + 8 * h;
    *reinterpret_cast<uint2*>(row + (((4 * qb + 2 * cc) ^ ds_row_swz) << 4)) = uint2{w.x, w.y};
    *reinterpret_cast<uint2*>(row + (((4 * qb + 2 * cc + 1) ^ ds_row_swz) << 4)) = uint2{w.z, w.w};
  };
  // dQ of one finished stage: this wave's 32 columns of the head dimension, all 64 queries,
  // summed over the key slices that hold a key some query of the stage may see
  auto dq_flush = [&](const char* tile, int q0) __attribute__((always_inline)) {
    const int keys = min(it.doc_end, q0 + kStep) - it.row0;
    const int cc_end = min(max((keys + 15) / 16, 0), kTile / 16);
    FragOffsets<kStep> fo_ds;      // the dS tile has rows of kStep elements
    fo_ds.init(lane);
    // the 2 x D / 32 blocks of 32 queries x 32 columns are dealt to the four waves
    constexpr int kBlocks = DB / 2;                      // per wave: 2 (D = 128), 1 (D = 64)
    const int db = DB == 4 ? wave : wave & 1;            // column block
    const int qb0 = DB == 4 ? 0 : wave >> 1;             // first (only) query block
    f32x16 acc[kBlocks];
#pragma unroll
    for (int b = 0; b < kBlocks; ++b) acc[b] = f32x16(0.f);
#pragma unroll 1
    for (int cc = 0; cc < cc_end; ++cc) {
      const bf16x8 kb = read_trans<D>(key_tile, fo, cc, db);
#pragma unroll
      for (int b = 0; b < kBlocks; ++b) {
        // offsets of query block qb0 + b (selected, not indexed: the table stays in registers)
        const int lo = (qb0 + b) ? fo_ds.trans[1][0] : fo_ds.trans[0][0];
        const int hi = (qb0 + b) ? fo_ds.trans[1][1] : fo_ds.trans[0][1];
        acc[b] = mfma(lds_read_tr8(tile + lo + cc * 16 * kStep * 2, tile + hi + cc * 16 * kStep * 2), kb, acc[b]);
      }
    }
    float* col = dq_acc_h + 32 * db + c;
#pragma unroll
    for (int b = 0; b < kBlocks; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = q0 + 32 * (qb0 + b) + 8 * (r / 4) + 4 * h + r % 4;
        if (row < it.doc_end) unsafeAtomicAdd(col + (size_t)row * Hq * D, acc[b][r]);
      }
  };

  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) { dkacc[i] = f32x16(0.f); dvacc[i] = f32x16(0.f); }

  // A 64-query stage against this wave's 32 keys: the two 32-query blocks are software-pipelined
  // by hand (this kernel runs one wave per SIMD, so nothing else hides LDS latency or overlaps
  // the exponentials with the matrix pipe):
  //   R0 | M1(0) + R1 | V(0) with M1(1) + T0 | M2(0) with V(1) + T1 | M2(1)
  // R: row-fragment and statistics reads, T: transposed-fragment reads, M1: S and dP,
  // V: P and dS on the vector ALU, M2: dV and dK.  Each matrix instruction is written next to
  // the vector and LDS work that should ride on it, and the fences keep that order.
  // MASKED: the stage touches the diagonal or runs past the document end (queries there are
  // clamped duplicates): P of a (query, key) pair outside the mask is set to exactly 0.
  auto stage = [&](const char* qt, const char* dot, const char* st, int q0, char* ds_tile, auto masked_c)
      __attribute__((always_inline)) {
    constexpr bool MASKED = decltype(masked_c)::value;
    constexpr int EPM = 16 / (2 * KK);  // score elements handled beside each matrix instruction
    bf16x8 qa[KK], da[KK], qb[KK], db_[KK];
    bf16x8 tq0[2][DB], td0[2][DB], tq1[2][DB], td1[2][DB];
    f32x4 l0[4], d0[4], l1[4], d1[4];
    // softmax of element r of one block: p = 2^(s cs - lse2), ds = p (dp - D)
    // (r stands for query q0 + 32 qb + 8 (r / 4) + 4 h + r % 4)
    const int t_lo = my_kv - q0 - 4 * h, t_hi = it.doc_end - q0 - 4 * h;   // allowed: t_lo <= 32 qb + 8 (r / 4) + r % 4 < t_hi
    auto soft = [&](f32x16& sv, const f32x16& dpv, f32x16& pv, const f32x4* l, const f32x4* dd, int r, int qb)
        __attribute__((always_inline)) {
      float e = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], cs, -l[r >> 2][r & 3]));
      if (MASKED) {
        const int t = 32 * qb + 8 * (r >> 2) + (r & 3);
        if (t < t_lo || t >= t_hi) e = 0.f;
      }
      pv[r] = e;
      sv[r] = e * (dpv[r] - dd[r >> 2][r & 3]);
    };
    // ---- R0
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qa[kk] = lds_read_frag(qt, fo.row_frag[kk]);
      da[kk] = lds_read_frag(dot, fo.row_frag[kk]);
    }
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      l0[rq] = *reinterpret_cast<const f32x4*>(st + (8 * rq + 4 * h) * 4);
      d0[rq] = *reinterpret_cast<const f32x4*>(st + 256 + (8 * rq + 4 * h) * 4);
    }
    __builtin_amdgcn_sched_barrier(0);
    // ---- M1(0) + R1
    f32x16 s0 = f32x16(0.f), dp0 = f32x16(0.f);
    static_for<KK>([&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      s0 = mfma(qa[kk], kf[kk], s0);
      qb[kk] = lds_read_frag(qt, fo.row_frag[kk] + 32 * D * 2);
      if (kk < 4) l1[kk] = *reinterpret_cast<const f32x4*>(st + (32 + 8 * kk + 4 * h) * 4);
      __builtin_amdgcn_sched_barrier(0);
      dp0 = mfma(da[kk], vf[kk], dp0);
      db_[kk] = lds_read_frag(dot, fo.row_frag[kk] + 32 * D * 2);
      if (kk < 4) d1[kk] = *reinterpret_cast<const f32x4*>(st + 256 + (32 + 8 * kk + 4 * h) * 4);
      __builtin_amdgcn_sched_barrier(0);
    });
    // ---- V(0) with M1(1) + T0
    f32x16 p0, s1 = f32x16(0.f), dp1 = f32x16(0.f);
    bf16x8 pb0[2], dsb0[2];
    static_for<KK>([&](auto kk_c) {
      constexpr int kk = decltype(kk_c)::value;
      s1 = mfma(qb[kk], kf[kk], s1);
#pragma unroll
      for (int e = 0; e < EPM; ++e) soft(s0, dp0, p0, l0, d0, EPM * 2 * kk + e, 0);
      td0[kk / DB][kk % DB] = read_trans<D>(dot, fo, kk / DB, kk % DB);
      __builtin_amdgcn_sched_barrier(0);
      dp1 = mfma(db_[kk], vf[kk], dp1);
#pragma unroll
      for (int e = 0; e < EPM; ++e) soft(s0, dp0, p0, l0, d0, EPM * (2 * kk + 1) + e, 0);
      tq0[kk / DB][kk % DB] = read_trans<D>(qt, fo, kk / DB, kk % DB);
      if ((kk + 1) * 2 * EPM % 8 == 0) {
        constexpr int i = (kk + 1) * 2 * EPM / 8 - 1;
        pb0[i] = pack8(p0, 8 * i);
        dsb0[i] = pack8(s0, 8 * i);
        if (FUSED) ds_store(ds_tile, dsb0[i], 0, i);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    // ---- M2(0) with V(1) + T1
    f32x16 p1;
    bf16x8 pb1[2], dsb1[2];
    static_for<2 * DB>([&](auto j_c) {
      constexpr int j = decltype(j_c)::value;
      dvacc[j % DB] = mfma(td0[j / DB][j % DB], pb0[j / DB], dvacc[j % DB]);
#pragma unroll
      for (int e = 0; e < EPM; ++e) soft(s1, dp1, p1, l1, d1, EPM * 2 * j + e, 1);
      td1[j / DB][j % DB] = read_trans<D>(dot + 32 * D * 2, fo, j / DB, j % DB);
      __builtin_amdgcn_sched_barrier(0);
      dkacc[j % DB] = mfma(tq0[j / DB][j % DB], dsb0[j / DB], dkacc[j % DB]);
#pragma unroll
      for (int e = 0; e < EPM; ++e) soft(s1, dp1, p1, l1, d1, EPM * (2 * j + 1) + e, 1);
      tq1[j / DB][j % DB] = read_trans<D>(qt + 32 * D * 2, fo, j / DB, j % DB);
      if ((j + 1) * 2 * EPM % 8 == 0) {
        constexpr int i = (j + 1) * 2 * EPM / 8 - 1;
        pb1[i] = pack8(p1, 8 * i);
        dsb1[i] = pack8(s1, 8 * i);
        if (FUSED) ds_store(ds_tile, dsb1[i], 1, i);
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    // ---- M2(1)
#pragma unroll
    for (int cc = 0; cc < 2; ++cc)
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        dvacc[db] = mfma(td1[cc][db], pb1[cc], dvacc[db]);
        dkacc[db] = mfma(tq1[cc][db], dsb1[cc], dkacc[db]);
      }
  };
  auto body = [&](int st, auto stage_c) {
    constexpr int ST = decltype(stage_c)::value;
    wait_vm<(NS - 2) * LPS>();
    __syncthreads();
    issue(st + NS - 1, (ST + NS - 1) % NS);
    const int step = it.step_begin + st;
    const int q0 = it.row0 + kStep * step;
    // fused: dQ of the previous stage, whose dS every wave has written before the barrier above
    if (FUSED && st > 0) dq_flush(ds_tiles + (1 - ST) * kDsBytes, q0 - kStep);
    if (!wave_active) return;
    const char* qt = smem + ST * kStageBytes;
    const char* dot = smem + (NS + ST) * kStageBytes;
    const char* stt = stat_base + ST * 4 * kStatBytes;
    if (q0 + kStep - 1 < wave_kv0) return;   // every query of the stage lies before this wave's keys
    char* ds_tile = ds_tiles + ST * kDsBytes;
    if (q0 < wave_kv0 + 32 || q0 + kStep > it.doc_end) stage(qt, dot, stt, q0, ds_tile, std::true_type{});
    else stage(qt, dot, stt, q0, ds_tile, std::false_type{});
  };
  for (;;) {
    restart();
#pragma unroll
    for (int st = 0; st < NS - 1; ++st) issue(st, st);
    for (int st = 0; st < n_steps; st += NS) {
      body(st, std::integral_constant<int, 0>{});
      if (st + 1 >= n_steps) break;
      body(st + 1, std::integral_constant<int, 1>{});
    }
    wait_vm<0>();  // nothing may still be landing in LDS when the workgroup goes on or retires
    if (FUSED) {       // dQ of the chain's last stage
      __syncthreads();
      dq_flush(ds_tiles + ((n_steps - 1) & 1) * kDsBytes, it.row0 + kStep * (it.step_begin + n_steps - 1));
    }
    if (--heads_left == 0) break;
    __syncthreads();   // every wave is done with the stages before they are refilled
    qbase += D; dobase += D; lse_h += N; dsum_h += N;
    if (FUSED) dq_acc_h += D;
  }

  if (it.slot >= 0) {
    float* part = partials + ((size_t)it.slot * Hq + head) * 2 * frag_floats<D>();
    store_frag<D>(part, dkacc, wave, lane);
    store_frag<D>(part + frag_floats<D>(), dvacc, wave, lane);
    return;
  }
  if (kv_valid) {
    store_rows<D>(dk + ((size_t)my_kv * Hkv + kvh) * D, dkacc, h, scale);
    store_rows<D>(dv + ((size_t)my_kv * Hkv + kvh) * D, dvacc, h, 1.0f);
  }
}

// Adds up fp32 partial fragments in a fixed order (chunks in chain order, then the q heads of
// the group) and stores bf16 rows.  NT tensors per partial (dQ: 1; [dK | dV]: 2), G partial
// heads per output head; tensor 0 is multiplied by `scale0`.  Elementwise: thread t owns
// float4 number t of the fragment.
template <int D, int NT>
__device__ __forceinline__ void sum_combine(int block, int n_items,
                                            const varlen_attn_combine_item* __restrict__ items,
                                            const float* __restrict__ partials,
                                            __bf16* __restrict__ out0, __bf16* __restrict__ out1,
                                            int Hin, int G, float scale0, int hpu = 1) {
  constexpr int DB = D / 32;
  constexpr int kBlocksPerItem = kTile * D / 4 / kThreads;
  const int Hout = Hin / G;
  const int sub = block % kBlocksPerItem;
  int rest = block / kBlocksPerItem;
  const int tensor = rest % NT; rest /= NT;
  const int idx = rest / Hout, oh = rest % Hout;
  if (idx >= n_items) return;
  const varlen_attn_combine_item it = items[idx];
  const int t = sub * kThreads + threadIdx.x;
  const int lane = t & 63, rq = (t >> 6) & 3, db = (t >> 8) % DB, wave = (t >> 8) / DB;
  const int h = lane >> 5, c = lane & 31;
  const int my_row = it.row0 + 32 * wave + c;
  if (my_row >= it.doc_end) return;
  const size_t psize = NT * frag_floats<D>();
  const float* p0 = partials + ((size_t)it.slot0 * Hin + oh * G) * psize + tensor * frag_floats<D>() +
                    (size_t)t * 4;
  // partial number j = ch * G + gh sits (ch * Hin + gh) partial sizes after the first; four
  // loads are kept in flight, the additions stay in index order (deterministic)
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  // of the G heads of a group only every hpu-th holds a partial (its unit swept hpu heads)
  const int Gp = G / hpu;
  const int n_parts = it.n_chunks * Gp;
  auto part = [&](int j) {
    return *reinterpret_cast<const f32x4*>(p0 + ((size_t)(j / Gp) * Hin + (j % Gp) * hpu) * psize);
  };
  int j = 0;
  for (; j + 4 <= n_parts; j += 4) {
    const f32x4 x0 = part(j), x1 = part(j + 1), x2 = part(j + 2), x3 = part(j + 3);
    acc += x0; acc += x1; acc += x2; acc += x3;
  }
  for (; j < n_parts; ++j) acc += part(j);
  const float mul = tensor == 0 ? scale0 : 1.0f;
  __bf16* out = tensor == 0 ? out0 : out1;
  *reinterpret_cast<uint2*>(out + ((size_t)my_row * Hout + oh) * D + 32 * db + 8 * rq + 4 * h) =
      pack4(acc[0] * mul, acc[1] * mul, acc[2] * mul, acc[3] * mul);
}

// The [dK | dV] reduction (over chunks and the q heads of a group); the dQ partials are summed
// at the end of the dK/dV kernel's grid.
template <int D>
__global__ void __launch_bounds__(kThreads)
bwd_combine_kernel(const varlen_attn_plan_header* __restrict__ hdr,
                   const varlen_attn_combine_item* __restrict__ col_items,
                   const float* __restrict__ col_partials, __bf16* __restrict__ dk,
                   __bf16* __restrict__ dv, int Hq, int Hkv, float scale) {
  sum_combine<D, 2>(blockIdx.x, hdr->n_col_combine, col_items, col_partials, dk, dv, Hq, Hq / Hkv, scale,
                    hdr->col_heads_per_unit);
}

}  // namespace

#endif  // VARLEN_ATTN_BWD_HPP_
