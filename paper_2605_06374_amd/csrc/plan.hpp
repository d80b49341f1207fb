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
//
// Units are placed longest first by cost class (kPlanClasses classes of equal width over the
// chunk lengths that occur): the hardware hands workgroups out in index order, so this is
// longest-job-first list scheduling.  The order inside a class is not defined.
//
// The kernel runs once per microbatch on a single compute unit, in front of everything else,
// so its latency is what counts: one thread per document, then one thread per tile (found by
// bisection in the running tile count of the documents), class counters per wave in LDS so that
// the same-address atomics of a wave stay inside the wave, and two sweeps over the tiles
// (count, then place) that run the same code.
// ----------------------------------------------------------------------------------------
constexpr int kPlanThreadsLarge = 1024;   // general form
constexpr int kPlanThreadsSmall = 64;     // one wave: every barrier is free, nothing is shared between waves
constexpr int kPlanClasses = 32;
constexpr int kMinChunkSteps = 4;
constexpr int kResidentGroups = 512;  // 256 CUs x 2 workgroups (forward, dQ)
constexpr int kTargetUnits = 512;   // (unit, head) pairs from cut chains to aim for: more cost partial-result traffic
constexpr long long kGroupSweepMinUnits = 512;  // column workgroups that must remain when units sweep several q heads
constexpr int kNoSplitSteps = 1 << 28;

struct PlanArgs {
  const int32_t* cu;
  int B, N, Hq, g, no_split;
  int force_ch[2];  // > 0: chunk length given by the caller (tuning), per direction
  int force_hpu;    // > 0: q heads per column unit given by the caller (a divisor of g)
  varlen_attn_plan_header* hdr;
  varlen_attn_unit* units[2];
  varlen_attn_combine_item* comb[2];
  int max_units, max_combine, max_slots[2], slots_cap;
  int32_t* status_copy;   // optional second place for the status word (device), or null
};

// inclusive sum over the lanes of a wave: data-parallel-primitive moves (shifts inside rows of
// 16 lanes, then the last lane of a row broadcast into the rows behind it), which cost a vector
// instruction each where a shuffle goes through the LDS crossbar and back
template <int kCtrl, int kRowMask>
__device__ __forceinline__ int dpp_or_zero(int v) {
  return __builtin_amdgcn_update_dpp(0, v, kCtrl, kRowMask, 0xF, false);
}
__device__ __forceinline__ int wave_inclusive_sum(int v) {
  v += dpp_or_zero<0x111, 0xF>(v);   // row_shr:1
  v += dpp_or_zero<0x112, 0xF>(v);   // row_shr:2
  v += dpp_or_zero<0x114, 0xF>(v);   // row_shr:4
  v += dpp_or_zero<0x118, 0xF>(v);   // row_shr:8
  v += dpp_or_zero<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_or_zero<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}
// value of lane `src` (wave-uniform) in every lane
__device__ __forceinline__ int lane_value(int v, int src) {
  return __builtin_amdgcn_readlane(v, __builtin_amdgcn_readfirstlane(src));
}

// Chunk length of direction d (0: row chains, 1: column chains) from the totals of the microbatch.
__device__ __forceinline__ int plan_chunk_steps(int d, unsigned long long steps_d, int n_tiles, int Hq,
                                                int forced) {
  const long long by_units = (long long)((steps_d * Hq + kTargetUnits - 1) / kTargetUnits);
  // Units of one head ~ steps / ch + tiles / 2 (a cut chain rarely divides evenly).  If
  // the tiles leave room, take the shortest chunks that keep every unit resident at once;
  // dK/dV partials are twice as large and its kernel is insensitive here: twice as long.
  const long long room = kResidentGroups / Hq - n_tiles / 2;
  long long by_fill = 0;
  if (room >= kResidentGroups / Hq / 4 && room > 0)
    by_fill = (d + 1) * (((long long)steps_d + room - 1) / room);
  const int ch = (int)max(max((long long)kMinChunkSteps, by_fill), by_units);
  return forced > 0 ? forced : ch;
}

// sum over the lanes of a wave (all lanes get it)
__device__ __forceinline__ int wave_total(int v) { return lane_value(wave_inclusive_sum(v), 63); }

// ----------------------------------------------------------------------------------------
// The u-th row unit of a microbatch of at most 64 documents and 256 tiles, in the order
// (tile, chunk), worked out by one wave from cu_seqlens alone with the plan's own rules (chunk
// length, nearly equal chunks, slots of cut tiles numbered in tile order): a forward workgroup
// of a small microbatch finds its unit this way instead of waiting for the plan.  All 64
// lanes must call it; every lane gets the same answer.  False: cu_seqlens is malformed (the
// plan reports it) or u is past the last unit.
// ----------------------------------------------------------------------------------------
constexpr int kSelfPlanDocs = 64, kSelfPlanTiles = 256;
__device__ __forceinline__ bool derive_row_unit(const int32_t* __restrict__ cu, int B, int N, int Hq,
                                                int no_split, int forced, int slots_cap, int u,
                                                int lane, varlen_attn_unit& out) {
  int s = 0, e = 0;
  if (lane < B) { s = cu[lane]; e = cu[lane + 1]; }
  const int l = e - s;
  const int cu_first = lane_value(s, 0), cu_last = lane_value(e, B - 1);
  if (__any(lane < B && l < 0) || cu_first != 0 || cu_last != N) return false;
  const int T = (l + kTile - 1) / kTile, S = (l + kStep - 1) / kStep;
  const int t_incl = wave_inclusive_sum(T);   // tiles up to and including this document
  const int n_tiles = lane_value(t_incl, 63);
  const int steps = wave_total(T * (T - 1) + S);
  int ch = no_split ? kNoSplitSteps : plan_chunk_steps(0, (unsigned long long)steps, n_tiles, Hq, forced);
  constexpr int kRounds = kSelfPlanTiles / 64;
  int ds[kRounds], de[kRounds], row0[kRounds], n[kRounds], nc[kRounds];
  // tiles 64 r + lane: their document (the first whose running tile count exceeds the tile
  // index, found by bisection over the lanes), first row and chain length
#pragma unroll
  for (int r = 0; r < kRounds; ++r) {
    ds[r] = de[r] = row0[r] = n[r] = 0;
    if (64 * r < n_tiles) {
      const int t = 64 * r + lane;
      // doc = number of documents whose running tile count is <= t (it is non-decreasing over
      // the lanes, and lane 63 holds n_tiles > t for every tile that exists)
      int doc = 0;
#pragma unroll
      for (int step = 32; step >= 1; step >>= 1)
        if (__shfl(t_incl, doc + step - 1) <= t) doc += step;
      ds[r] = __shfl(s, doc); de[r] = __shfl(e, doc);
      const int before = __shfl(t_incl - T, doc);
      row0[r] = ds[r] + (t - before) * kTile;
      n[r] = t < n_tiles ? (min(row0[r] + kTile, de[r]) - 1 - ds[r]) / kStep + 1 : 0;
    }
  }
  // chunks per tile; the chunk length doubles until the chunks of cut chains fit their slots
#pragma unroll 1
  for (;;) {
    int cut = 0;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      nc[r] = n[r] ? (n[r] + ch - 1) / ch : 0;
      cut += nc[r] > 1 ? nc[r] : 0;
    }
    if (no_split || wave_total(cut) <= slots_cap) break;
    ch *= 2;
  }
  int units_before = 0, slots_before = 0;
#pragma unroll
  for (int r = 0; r < kRounds; ++r) {
    if (64 * r < n_tiles) {
      const int cut = nc[r] > 1 ? nc[r] : 0;
      const int u_incl = wave_inclusive_sum(nc[r]), s_incl = wave_inclusive_sum(cut);
      const int u0 = units_before + u_incl - nc[r];
      const unsigned long long hit = __ballot(u0 <= u && u < u0 + nc[r]);
      if (hit) {
        const int src = __ffsll((long long)hit) - 1;
        const int nn = lane_value(n[r], src), k = lane_value(nc[r], src), c = u - lane_value(u0, src);
        const int slot0 = slots_before + lane_value(s_incl - cut, src);
        const int base = nn / k, rem = nn % k;
        const int first = c * base + min(c, rem), len = base + (c < rem ? 1 : 0);
        out = varlen_attn_unit{lane_value(row0[r], src), lane_value(ds[r], src), lane_value(de[r], src), first,
                               first + len, k > 1 ? slot0 + c : -1, len, 0};
        return true;
      }
      units_before += lane_value(u_incl, 63);
      slots_before += lane_value(s_incl, 63);
    }
  }
  return false;
}

template <int kPlanThreads>
__device__ __forceinline__ void plan_body(const PlanArgs& a) {
  constexpr int kPlanWaves = kPlanThreads / 64;
  // one wave: the tiles are visited in order, so the slots of cut row chains can be numbered in
  // tile order by a running sum (a forward workgroup that works out its own unit needs that)
  constexpr bool kOrdered = kPlanWaves == 1;
  static_assert(2 * kPlanClasses * kPlanWaves == kPlanThreads, "one thread per class counter");
  __shared__ int doc_first_tile[kPlanThreads + 1];  // running tile count of the batch's documents
  __shared__ int doc_s[kPlanThreads], doc_e[kPlanThreads];
  __shared__ int hist[2][kPlanClasses][kPlanWaves];    // units per (direction, class, wave), then cursors
  __shared__ int class_total[2][kPlanClasses];
  __shared__ int wave_sum[kPlanWaves];
  __shared__ unsigned long long pairs, steps[2];
  __shared__ int n_tiles, bad, max_chain[2];
  __shared__ int split[2], n_units[2], n_slots[2], n_comb[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int32_t* cu = a.cu;
  if (tid == 0) {
    bad = (cu[0] != 0) || (cu[a.B] != a.N);
    pairs = steps[0] = steps[1] = 0;
    n_tiles = 0;
  }
  if (tid < 2) split[tid] = n_units[tid] = n_slots[tid] = n_comb[tid] = max_chain[tid] = 0;
  __syncthreads();
  // ---- totals over the documents: pairs, steps of both directions, tiles, longest chains
  {
    unsigned long long my_pairs = 0, my_r = 0, my_c = 0;
    int my_bad = 0, my_tiles = 0, my_max = 0;
#pragma unroll 1
    for (int b = tid; b < a.B; b += kPlanThreads) {
      const long long l = (long long)cu[b + 1] - cu[b];
      if (l < 0) { my_bad = 1; continue; }
      my_pairs += (unsigned long long)(l * (l + 1) / 2);
      const long long T = (l + kTile - 1) / kTile, S = (l + kStep - 1) / kStep;
      my_r += (unsigned long long)(T * (T - 1) + S);
      my_c += (unsigned long long)(T * S - T * (T - 1));
      my_tiles += (int)T;
      my_max = max(my_max, (int)S);
    }
    if (my_bad) bad = 1;
    if (my_pairs) {
      atomicAdd(&pairs, my_pairs); atomicAdd(&steps[0], my_r); atomicAdd(&steps[1], my_c);
      atomicAdd(&n_tiles, my_tiles);
      atomicMax(&max_chain[0], my_max);   // the longest row and column chains are both ceil(l / 64)
    }
  }
  __syncthreads();
  varlen_attn_plan_header* hdr = a.hdr;
  if (bad) {
    if (tid < (int)(sizeof(varlen_attn_plan_header) / 4)) reinterpret_cast<int32_t*>(hdr)[tid] = 0;
    __syncthreads();
    if (tid == 0) {
      hdr->status = VARLEN_ATTN_BAD_CU_SEQLENS;
      if (a.status_copy) *a.status_copy = VARLEN_ATTN_BAD_CU_SEQLENS;
    }
    return;
  }
  int ch[2];
#pragma unroll
  for (int d = 0; d < 2; ++d) {
    ch[d] = kNoSplitSteps;
    if (!a.no_split) {
      ch[d] = plan_chunk_steps(d, steps[d], n_tiles, a.Hq, a.force_ch[d]);
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
  const int longest = max_chain[0];

  // mode 0: count the units of every cost class (and the chunks of cut chains); mode 1: place.
  int mode = 0, shift[2] = {0, 0};
#pragma unroll 1
  for (;;) {
    if (mode == 0) {
#pragma unroll
      for (int d = 0; d < 2; ++d) {
        shift[d] = 0;
        while ((min(ch[d], longest) - 1) >> shift[d] >= kPlanClasses) ++shift[d];
      }
      reinterpret_cast<int*>(hist)[tid] = 0;   // 2 x 32 x waves counters: one per thread
      if (tid < 2) split[tid] = 0;
      __syncthreads();
    }
    int row_slots_before = 0;   // cut row chains' slots so far, in tile order (single-wave form)
#pragma unroll 1
    for (int b0 = 0; b0 < a.B; b0 += kPlanThreads) {
      // ---- this batch's documents: running tile count (exclusive) by a workgroup-wide scan
      {
        const int b = b0 + tid;
        int s = 0, e = 0;
        if (b < a.B) { s = cu[b]; e = cu[b + 1]; }
        const int T = (e - s + kTile - 1) / kTile;
        const int incl = wave_inclusive_sum(T);
        if (lane == 63) wave_sum[wave] = incl;
        doc_s[tid] = s; doc_e[tid] = e;
        __syncthreads();
        int before = 0;
#pragma unroll 1
        for (int w = 0; w < wave; ++w) before += wave_sum[w];
        doc_first_tile[tid + 1] = before + incl;
        if (tid == 0) doc_first_tile[0] = 0;
        __syncthreads();
      }
      const int batch_tiles = doc_first_tile[kPlanThreads];
      // every thread makes the same number of turns (the running sums are wave-wide scans)
#pragma unroll 1
      for (int t0 = 0; t0 < batch_tiles; t0 += kPlanThreads) {
        const int t = t0 + tid;
        const bool valid = t < batch_tiles;
        int ss = 0, ee = 0, row0 = 0, n_d[2] = {0, 0}, nc_d[2] = {0, 0};
        if (valid) {
          // document of tile t: the last one whose first tile is <= t (documents without tiles
          // repeat the value of their successor and are skipped by taking the last)
          int lo = 0, hi = kPlanThreads;   // doc_first_tile[lo] <= t < doc_first_tile[hi]
#pragma unroll 1
          while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (doc_first_tile[mid] <= t) lo = mid; else hi = mid;
          }
          ss = doc_s[lo]; ee = doc_e[lo];
          row0 = ss + (t - doc_first_tile[lo]) * kTile;
          n_d[0] = (min(row0 + kTile, ee) - 1 - ss) / kStep + 1;
          n_d[1] = (ee - row0 + kStep - 1) / kStep;
          nc_d[0] = (n_d[0] + ch[0] - 1) / ch[0];
          nc_d[1] = (n_d[1] + ch[1] - 1) / ch[1];
        }
        // slots of a cut row chain, numbered in tile order
        int ordered_slot0 = 0;
        if (kOrdered) {
          const int cut = nc_d[0] > 1 ? nc_d[0] : 0;
          const int incl = wave_inclusive_sum(cut);
          ordered_slot0 = row_slots_before + incl - cut;
          row_slots_before += lane_value(incl, 63);
        }
        if (valid) {
#pragma unroll
          for (int d = 0; d < 2; ++d) {
            const int n = n_d[d], nc = nc_d[d], base = n / nc, rem = n % nc;
            // nc - rem chunks of `base` steps, rem chunks of base + 1 (those come first in the chain)
            int* h_lo = &hist[d][(base - 1) >> shift[d]][wave];
            int* h_hi = &hist[d][base >> shift[d]][wave];
            if (mode == 0) {
              atomicAdd(h_lo, nc - rem);
              if (rem) atomicAdd(h_hi, rem);
              if (nc > 1) atomicAdd(&split[d], nc);
            } else {
              int slot0 = -1;
              if (nc > 1 || (d == 1 && a.g > hpu)) {
                if (kOrdered && d == 0) { slot0 = ordered_slot0; atomicAdd(&n_slots[0], nc); }
                else slot0 = atomicAdd(&n_slots[d], nc);
                const int ci = atomicAdd(&n_comb[d], 1);
                if (ci < a.max_combine && slot0 + nc <= a.max_slots[d])
                  a.comb[d][ci] = varlen_attn_combine_item{row0, ee, slot0, nc};
              }
              int pos_lo = atomicAdd(h_lo, nc - rem);
              int pos_hi = rem ? atomicAdd(h_hi, rem) : 0;
#pragma unroll 1
              for (int c = 0; c < nc; ++c) {
                const int first = c * base + min(c, rem), len = base + (c < rem ? 1 : 0);
                const int pos = c < rem ? pos_hi++ : pos_lo++;
                if (pos < a.max_units)
                  a.units[d][pos] = varlen_attn_unit{row0, ss, ee, first, first + len,
                                                     slot0 < 0 ? -1 : slot0 + c, len, 0};
              }
            }
          }
        }
      }
      __syncthreads();   // the batch arrays are rewritten by the next batch
    }
    if (mode == 1) break;
    // lengthen the chunks until the cut chains fit their slots
    const bool fit0 = split[0] <= a.slots_cap, fit1 = split[1] <= a.slots_cap;
    if (!(fit0 && fit1)) {
      __syncthreads();
      if (!fit0) ch[0] *= 2;
      if (!fit1) ch[1] *= 2;
      continue;
    }
    // counters -> start positions: classes from the longest down, waves in order inside a class
    {
      const int d = tid / (kPlanClasses * kPlanWaves), cls = (tid / kPlanWaves) % kPlanClasses,
                w = tid % kPlanWaves;
      const int own = hist[d][cls][w];
      int incl = own;   // inclusive sum over the 16 waves of this class (16 adjacent lanes)
#pragma unroll
      for (int off = 1; off < kPlanWaves; off <<= 1) {
        const int o = __shfl_up(incl, off);
        if (w >= off) incl += o;
      }
      if (w == kPlanWaves - 1) class_total[d][cls] = incl;
      __syncthreads();
      int above = 0;
#pragma unroll 1
      for (int c2 = cls + 1; c2 < kPlanClasses; ++c2) above += class_total[d][c2];
      if (cls == 0 && w == kPlanWaves - 1) n_units[d] = above + incl;
      __syncthreads();
      hist[d][cls][w] = above + incl - own;
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
    if (a.status_copy) *a.status_copy = hdr->status;
    hdr->n_row_units = ok ? n_units[0] : 0;
    hdr->n_col_units = ok ? n_units[1] : 0;
    hdr->n_row_combine = ok ? n_comb[0] : 0;
    hdr->n_col_combine = ok ? n_comb[1] : 0;
    hdr->row_chunk_steps = ch[0];
    hdr->col_chunk_steps = ch[1];
    hdr->n_row_slots = n_slots[0];
    hdr->n_col_slots = n_slots[1];
    hdr->row_class_shift = shift[0];
    hdr->col_heads_per_unit = hpu;
    hdr->col_class_shift = shift[1];
    for (int i = 0; i < 2; ++i) hdr->reserved[i] = 0;
    hdr->pairs = (int64_t)pairs;
  }
}

template <int kPlanThreads>
__global__ void __launch_bounds__(kPlanThreads) plan_kernel(PlanArgs a) {
  plan_body<kPlanThreads>(a);
}

}  // namespace

#endif  // VARLEN_ATTN_PLAN_HPP_
