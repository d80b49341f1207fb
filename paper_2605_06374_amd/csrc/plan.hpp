// Plan kernel: cu_seqlens -> validated, chunked work units (integer work only).
#ifndef VARLEN_ATTN_PLAN_HPP_
#define VARLEN_ATTN_PLAN_HPP_

#include "tiles.hpp"

namespace {

// ----------------------------------------------------------------------------------------
// Plan: cu_seqlens -> validated work units (integer work only).
//
// One workgroup.  For both directions (0: row chains for forward / dQ, 1: column chains for
// dK / dV) it picks the chunk length, cuts every tile's chain into nearly equal chunks and
// writes the units.  Chunk length: at least kMinChunkSteps; on a microbatch whose tiles do not
// fill the GPU by themselves, just long enough that all (unit, head) pairs are resident at
// once (kResidentGroups workgroups: one round, no second wave of stragglers); otherwise long
// enough that about kTargetUnits pairs exist; and always such that the partial-result slots
// fit the workspace.
// Small microbatches (every unit is short anyway) are written in sweep order; large ones are
// placed by a counting sort on cost, descending (longest job first).
//
// The kernel runs once per microbatch on a single compute unit with a cold instruction
// cache, so its latency follows the amount of code it executes: the two directions and the
// two passes share one copy of the per-tile code (loops deliberately not unrolled).
// ----------------------------------------------------------------------------------------
constexpr int kPlanThreads = 1024;
constexpr int kPlanBins = 1024;
constexpr int kMinChunkSteps = 4;
constexpr int kResidentGroups = 512;  // 256 CUs x 2 workgroups (forward, dQ)
constexpr int kTargetUnits = 512;   // (unit, head) pairs from cut chains to aim for: more cost partial-result traffic
constexpr long long kGroupSweepMinUnits = 512;  // column workgroups that must remain when units sweep several q heads
constexpr int kNoSplitSteps = 1 << 28;
constexpr long long kSortAboveSteps = 1024;  // (tile step, head) pairs; below: sweep order

struct PlanArgs {
  const int32_t* cu;
  int B, N, Hq, g, shift, no_split;
  int force_ch[2];
  int force_hpu;    // > 0: q heads per column unit given by the caller (a divisor of g)  // > 0: chunk length given by the caller (tuning), per direction
  varlen_attn_plan_header* hdr;
  varlen_attn_unit* units[2];
  varlen_attn_combine_item* comb[2];
  int max_units, max_combine, max_slots[2], slots_cap;
};

__global__ void __launch_bounds__(kPlanThreads) plan_kernel(PlanArgs a) {
  __shared__ int bad;
  __shared__ int hist[2][kPlanBins];    // units per cost bucket, then start offsets
  __shared__ int cursor[2][kPlanBins];
  __shared__ int wsum[kPlanThreads / 64];
  __shared__ unsigned long long pairs, steps[2];
  __shared__ int n_tiles;
  __shared__ int split[2], n_units[2], n_slots[2], n_comb[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* cu = a.cu;
  if (tid == 0) {
    bad = (cu[0] != 0) || (cu[a.B] != a.N);
    pairs = steps[0] = steps[1] = 0;
    n_tiles = 0;
  }
  if (tid < 2) split[tid] = n_units[tid] = n_slots[tid] = n_comb[tid] = 0;
  __syncthreads();
  {
    unsigned long long my_pairs = 0, my_r = 0, my_c = 0;
    int my_bad = 0, my_tiles = 0;
#pragma unroll 1
    for (int b = tid; b < a.B; b += kPlanThreads) {
      const long long l = (long long)cu[b + 1] - cu[b];
      if (l < 0) { my_bad = 1; continue; }
      my_pairs += (unsigned long long)(l * (l + 1) / 2);
      const long long T = (l + kTile - 1) / kTile, S = (l + kStep - 1) / kStep;
      my_r += (unsigned long long)(T * (T - 1) + S);
      my_c += (unsigned long long)(T * S - T * (T - 1));
      my_tiles += (int)T;
    }
    if (my_bad) bad = 1;
    if (my_pairs) { atomicAdd(&pairs, my_pairs); atomicAdd(&steps[0], my_r); atomicAdd(&steps[1], my_c); atomicAdd(&n_tiles, my_tiles); }
  }
  __syncthreads();
  varlen_attn_plan_header* hdr = a.hdr;
  if (bad) {
    if (tid < (int)(sizeof(varlen_attn_plan_header) / 4)) reinterpret_cast<int32_t*>(hdr)[tid] = 0;
    __syncthreads();
    if (tid == 0) hdr->status = VARLEN_ATTN_BAD_CU_SEQLENS;
    return;
  }
  const bool sorted = (long long)steps[0] * a.Hq > kSortAboveSteps;
  int ch[2];
#pragma unroll
  for (int d = 0; d < 2; ++d) {
    ch[d] = kNoSplitSteps;
    if (!a.no_split) {
      // 2 * steps / ch bounds the slots of the chains that get cut (each has > ch steps)
      const long long by_units = (long long)((steps[d] * a.Hq + kTargetUnits - 1) / kTargetUnits);
      const long long by_slots = (long long)((2 * steps[d] + a.slots_cap - 1) / a.slots_cap);
      // Units of one head ~ steps / ch + tiles / 2 (a cut chain rarely divides evenly).  If
      // the tiles leave room, take the shortest chunks that keep every unit resident at once;
      // dK/dV partials are twice as large and its kernel is insensitive here: twice as long.
      const long long room = kResidentGroups / a.Hq - n_tiles / 2;
      long long by_fill = 0;
      if (room >= kResidentGroups / a.Hq / 4 && room > 0)
        by_fill = (d + 1) * (((long long)steps[d] + room - 1) / room);
      const long long floor_ch = max((long long)kMinChunkSteps, by_fill);
      ch[d] = (int)max(floor_ch, sorted ? by_units : max(by_units, by_slots));
      if (a.force_ch[d] > 0) ch[d] = (int)max((long long)a.force_ch[d], sorted ? 1 : by_slots);
    }
  }
  // Grouped-query attention: a column unit may sweep several q heads of its group (their dK,
  // dV add up in its registers: fewer and smaller group sums afterwards) as long as enough
  // workgroups remain.  Units of one head ~ steps / ch + tiles / 2.
  int hpu = 1;
  if (a.g > 1) {
    if (a.force_hpu > 0 && a.g % a.force_hpu == 0) {
      hpu = a.force_hpu;
    } else if (!a.no_split) {   // unsplit plans must not depend on the rest of the microbatch
      const long long groups = ((long long)steps[1] / ch[1] + n_tiles / 2) * a.Hq;
      for (int cand = 2; cand <= a.g; ++cand)
        if (a.g % cand == 0 && groups / cand >= kGroupSweepMinUnits) hpu = cand;
    }
  }
  if (sorted) {
    hist[0][tid] = hist[1][tid] = 0;
    cursor[0][tid] = cursor[1][tid] = 0;
  }
  __syncthreads();

  // mode 0: count unit costs (sorted plans only); mode 1: write units.
  int mode = sorted ? 0 : 1;
#pragma unroll 1
  for (;;) {
    // Every (document, tile) once per direction: the lower half of the waves makes the row
    // units, the upper half the column units.  The waves of a half walk all batches of 64
    // documents; tile 0 of a document is taken by one lane of the wave that owns the batch,
    // and the further tiles of longer documents are swept by whole waves, the long documents
    // dealt round-robin to the waves of the half.  One call site for the per-tile code.
    constexpr int kHalfWaves = kPlanThreads / 64 / 2;
    const int d = wave / kHalfWaves, hw = wave % kHalfWaves;
    int long_rank = 0;
#pragma unroll 1
    for (int b0 = 0; b0 < a.B; b0 += 64) {
      const int b = b0 + lane;
      int s = 0, e = 0;
      if (b < a.B) { s = cu[b]; e = cu[b + 1]; }
      const int T = (e - s + kTile - 1) / kTile;
      unsigned long long pending = __ballot(T > 1);
      const bool own_batch = ((b0 >> 6) % kHalfWaves) == hw;
      int ss = s, ee = e, i = 0, TT = own_batch ? min(T, 1) : 0;
#pragma unroll 1
      for (;;) {
#pragma unroll 1
        while (__any(i < TT)) {
          if (i < TT) {
            const int row0 = ss + i * kTile;
            {
              const int n = d == 0 ? (min(row0 + kTile, ee) - 1 - ss) / kStep + 1
                                   : (ee - row0 + kStep - 1) / kStep;
              const int nc = (n + ch[d] - 1) / ch[d], base = n / nc, rem = n % nc;
              if (mode == 0) {
                atomicAdd(&hist[d][(base - 1) >> a.shift], nc - rem);
                if (rem) atomicAdd(&hist[d][base >> a.shift], rem);
                if (nc > 1) atomicAdd(&split[d], nc);
              } else {
                int slot0 = -1;
                if (nc > 1 || (d == 1 && a.g > hpu)) {
                  slot0 = atomicAdd(&n_slots[d], nc);
                  const int ci = atomicAdd(&n_comb[d], 1);
                  if (ci < a.max_combine && slot0 + nc <= a.max_slots[d])
                    a.comb[d][ci] = varlen_attn_combine_item{row0, ee, slot0, nc};
                }
                int pos0 = sorted ? 0 : atomicAdd(&n_units[d], nc);
#pragma unroll 1
                for (int c = 0; c < nc; ++c) {
                  const int b_ = c * base + min(c, rem), len = base + (c < rem ? 1 : 0);
                  int pos = pos0 + c;
                  if (sorted) {
                    const int k = (len - 1) >> a.shift;
                    pos = hist[d][k] + atomicAdd(&cursor[d][k], 1);
                  }
                  if (pos < a.max_units)
                    a.units[d][pos] = varlen_attn_unit{row0, ss, ee, b_, b_ + len,
                                                       slot0 < 0 ? -1 : slot0 + c, len, 0};
                }
              }
            }
          }
          i += 64;
        }
        // next long document dealt to this wave
        bool found = false;
#pragma unroll 1
        while (pending && !found) {
          const int src = __ffsll((long long)pending) - 1;
          pending &= pending - 1;
          if ((long_rank++ % kHalfWaves) == hw) {
            ss = __shfl(s, src); ee = __shfl(e, src); TT = __shfl(T, src);
            i = 1 + lane;
            found = true;
          }
        }
        if (!found) break;
      }
    }
    __syncthreads();
    if (mode == 1) break;
    // sorted plans: lengthen the chunks until the cut chains fit, then turn the histograms
    // into start offsets (exclusive suffix sums: longest first)
    const bool fit0 = split[0] <= a.slots_cap, fit1 = split[1] <= a.slots_cap;
    __syncthreads();
    if (!(fit0 && fit1)) {
      if (!fit0) ch[0] *= 2;
      if (!fit1) ch[1] *= 2;
      hist[0][tid] = hist[1][tid] = 0;
      if (tid < 2) split[tid] = 0;
      __syncthreads();
      continue;
    }
#pragma unroll 1
    for (int d = 0; d < 2; ++d) {
      const int own = hist[d][tid];
      int v = own;
#pragma unroll 1
      for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_down(v, off);
        if (lane + off < 64) v += o;
      }
      if (lane == 0) wsum[wave] = v;
      __syncthreads();
      int above = 0, total = 0;
#pragma unroll 1
      for (int w = 0; w < kPlanThreads / 64; ++w) {
        const int x = wsum[w];
        total += x;
        if (w > wave) above += x;
      }
      hist[d][tid] = v - own + above;
      if (tid == 0) n_units[d] = total;
      __syncthreads();
    }
    mode = 1;
  }
  if (tid == 0) {
    // The capacities are worst-case bounds (tiles <= N / 128 + B; a cut chain of n > ch steps
    // takes ceil(n / ch) <= 2 n / ch chunks, and ch was lengthened until those fit), so this
    // cannot fail; if it ever does, it is an error of its own and nothing is planned.
    const bool ok = n_units[0] <= a.max_units && n_units[1] <= a.max_units &&
                    n_comb[0] <= a.max_combine && n_comb[1] <= a.max_combine &&
                    n_slots[0] <= a.max_slots[0] && n_slots[1] <= a.max_slots[1];
    hdr->status = ok ? VARLEN_ATTN_OK : VARLEN_ATTN_PLAN_OVERFLOW;
    hdr->n_row_units = ok ? n_units[0] : 0;
    hdr->n_col_units = ok ? n_units[1] : 0;
    hdr->n_row_combine = ok ? n_comb[0] : 0;
    hdr->n_col_combine = ok ? n_comb[1] : 0;
    hdr->row_chunk_steps = ch[0];
    hdr->col_chunk_steps = ch[1];
    hdr->n_row_slots = n_slots[0];
    hdr->n_col_slots = n_slots[1];
    hdr->sorted = sorted;
    hdr->col_heads_per_unit = hpu;
    for (int i = 0; i < 3; ++i) hdr->reserved[i] = 0;
    hdr->pairs = (int64_t)pairs;
  }
}

}  // namespace

#endif  // VARLEN_ATTN_PLAN_HPP_
