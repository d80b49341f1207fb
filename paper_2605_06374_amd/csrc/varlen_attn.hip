// Document-masked causal attention, forward and backward, for packed variable-length
// microbatches on MI355X (gfx950 / CDNA4).  Hand-written HIP; wave64; bf16 MFMA
// (v_mfma_f32_32x32x16_bf16) with fp32 accumulation.
//
// The operation is the quadratic term of the micro-batch time model (Section 5.2, Eq. 1):
// documents of lengths l_1..l_k packed into N tokens, block-diagonal mask, causal inside
// each block.  Only (query tile, key tile) pairs that contain an allowed (t, j) are ever
// visited, so the work follows sum l_i^2, not N^2.
//
// Register/lane conventions used by every kernel below (L = lane, h = L / 32, c = L % 32):
//   MFMA 32x32x16:  A[i][k]: lane holds i = c, k = 8h + e (e = 0..7)
//                   B[k][j]: lane holds j = c, k = 8h + e
//                   C[i][j]: lane holds j = c, i = 8 (r / 4) + 4h + r % 4 (r = 0..15)
// The kernels always put the softmax row index on the lane (j = c) so that row statistics
// are per-lane scalars, and feed the exponentiated scores straight back as a B operand:
// registers 8cc..8cc+7 of a C tile are the k positions of the cc-th 16-deep slice, standing
// for rows 16cc + 4h + {0..3} and 16cc + 8 + 4h + {0..3}.  The matching A operand is a
// transposed read of a row-major LDS tile (ds_read_b64_tr_b16, twice).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>
#include <utility>
#include <mutex>
#include <vector>

#include "varlen_attn.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kTile = VARLEN_ATTN_TILE_ROWS;  // rows of a work item (4 waves x 32)
constexpr int kStep = VARLEN_ATTN_STEP_ROWS;  // rows staged per iteration of a chain
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleTau = 8.0f;  // running max may lag by up to 2^8 before O is rescaled

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose body may hold
// scheduling fences (an ordinary loop that holds one is not unrolled).
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// ----------------------------------------------------------------------------------------
// LDS tiles: row-major [rows][D] bf16, addressed in 16-byte chunks with an XOR swizzle that
// keeps both the row-fragment reads (ds_read_b128, 32 rows x one chunk) and the transposed
// reads (ds_read_b64_tr_b16, 4 rows x 64 bytes per half-wave) spread over the banks.
// ----------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ int swz(int row) {
  if constexpr (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  else return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
}
template <int D>
__device__ __forceinline__ int chunk_off(int row, int chunk) {  // in bytes
  return (row * (D / 8) + (chunk ^ swz<D>(row))) * 16;
}

__device__ __forceinline__ bf16x8 lds_read_frag(const char* tile, int byte_off) {
  return *reinterpret_cast<const bf16x8*>(tile + byte_off);
}

// Transposed 4x(16 lanes) read: lane i of each 16-lane group passes the address of 4
// consecutive columns of row (i / 4); it receives rows 0..3 at column i of the group.
__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// value held by the same column in the other half of the wave (lane ^ 32), combined by op
__device__ __forceinline__ float half_max(float x) {
  unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_fmaxf(__builtin_bit_cast(float, (unsigned)r[0]),
                         __builtin_bit_cast(float, (unsigned)r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int first) {
  bf16x8 out;
#pragma unroll
  for (int e = 0; e < 8; e += 2) {
    f32x2 t = {v[first + e], v[first + e + 1]};
    bf16x2 b = __builtin_convertvector(t, bf16x2);
    out[e] = b[0];
    out[e + 1] = b[1];
  }
  return out;
}

__device__ __forceinline__ uint2 pack4(float a, float b, float c, float d) {
  f32x2 t0 = {a, b}, t1 = {c, d};
  bf16x2 b0 = __builtin_convertvector(t0, bf16x2), b1 = __builtin_convertvector(t1, bf16x2);
  return uint2{__builtin_bit_cast(unsigned, b0), __builtin_bit_cast(unsigned, b1)};
}

// ----------------------------------------------------------------------------------------
// Global -> LDS staging without registers (global_load_lds_dwordx4): the 64 lanes of a wave
// write 1 KiB contiguous in LDS starting at the wave-uniform address in M0, each lane taking
// its 16 bytes from its own global address.  A stage holds kSub = 32 rows of a [rows][D] tile;
// the XOR swizzle is applied on the global side (lane of physical chunk pc in row r fetches
// logical chunk pc ^ swz(r)).  Rows past `row_last` are clamped to it: they are finite
// duplicates that the causal mask (or a zero P) removes, never garbage.
//
// The loads are invisible to the compiler's wait-count bookkeeping (inline asm), which is
// the point: a compiler-inserted wait would be vmcnt(0) before every LDS read.  The kernels
// wait explicitly with wait_vm<N>() and publish with a barrier.  Extra outstanding loads can
// only make compiler-inserted vmcnt waits longer, never too short (in-order completion).
// ----------------------------------------------------------------------------------------
constexpr int kSub = 32;  // rows per pipeline stage

// base: wave-uniform 64-bit address; voff: this lane's unsigned byte offset from it
__device__ __forceinline__ void dma16(unsigned long long base, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(base), "s"(lds_addr)
               : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt immediate");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// vmcnt(0) as an instruction the compiler's wait-count pass can see (expcnt, lgkmcnt untouched)
__device__ __forceinline__ void wait_all_vm_visible() { __builtin_amdgcn_s_waitcnt(0x0F70); }
__device__ __forceinline__ unsigned lds_addr_of(const void* p) {
  return (unsigned)(size_t)(const __attribute__((address_space(3))) char*)p;
}
__device__ __forceinline__ unsigned long long uniform64(const void* p) {
  const unsigned long long v = (unsigned long long)(size_t)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return ((unsigned long long)hi << 32) | lo;
}

// Loads 32-row stages of a [rows][D] bf16 tile whose rows are `stride_bytes` apart.  The
// per-lane part of the address is a 32-bit offset fixed at init; the stage's first row goes
// into the wave-uniform base, so a stage costs no vector arithmetic unless it runs past
// `row_last` (then rows are clamped lane by lane).
template <int D, int ROWS = kSub>
struct StageLoader {
  static constexpr int kRowsPerInstr = 1024 / (D * 2);      // 4 (D=128), 8 (D=64)
  static constexpr int kInstr = ROWS / kRowsPerInstr;       // wave-level loads per stage
  static constexpr int kPerWave = kInstr / 4;               // 4 waves share a stage
  int row_in_stage[kPerWave];
  unsigned col_bytes[kPerWave];
  unsigned voff[kPerWave];
  unsigned stride_bytes;
  __device__ __forceinline__ void init(int wave, int lane, unsigned stride_bytes_) {
    stride_bytes = stride_bytes_;
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const int j = wave + 4 * i;
      const int r = kRowsPerInstr * j + lane / (D / 8), pc = lane % (D / 8);
      row_in_stage[i] = r;
      col_bytes[i] = (unsigned)((pc ^ swz<D>(r)) * 16);
      voff[i] = (unsigned)r * stride_bytes + col_bytes[i];
    }
  }
  // tile rows [row0, row0 + ROWS) of `base` -> LDS at `lds`; rows above row_last are clamped
  __device__ __forceinline__ void issue(const __bf16* base, int row0, int row_last, unsigned lds,
                                        int wave) const {
    const unsigned long long b =
        uniform64(reinterpret_cast<const char*>(base) + (size_t)row0 * stride_bytes);
    if (row0 + ROWS - 1 <= row_last) {
#pragma unroll
      for (int i = 0; i < kPerWave; ++i)
        dma16(b, voff[i], __builtin_amdgcn_readfirstlane(lds + (wave + 4 * i) * 1024));
    } else {
#pragma unroll
      for (int i = 0; i < kPerWave; ++i) {
        const int r = min(row_in_stage[i], row_last - row0);   // row_last >= row0 always
        dma16(b, (unsigned)r * stride_bytes + col_bytes[i],
              __builtin_amdgcn_readfirstlane(lds + (wave + 4 * i) * 1024));
      }
    }
  }
};

// 64 consecutive floats (clamped at index `last`) -> 256 bytes of LDS, one wave-level load
__device__ __forceinline__ void dma_floats64(const float* base, int first, int last, unsigned lds,
                                             int lane) {
  const unsigned long long b = uniform64(base + first);
  unsigned voff = (unsigned)lane * 4;
  if (first + 63 > last) voff = (unsigned)min(lane, last - first) * 4;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
               :
               : "v"(voff), "s"(b), "s"(__builtin_amdgcn_readfirstlane(lds))
               : "memory");
}

// per-lane byte offsets (inside a stage) of the two kinds of fragment reads
template <int D>
struct FragOffsets {
  int row_frag[D / 16];     // A/B row fragment of row c, k slice kk: chunk 2kk + h
  int trans[D / 32][2];     // transposed fragment, column block db, rows 4h + i/4 (+8)
  __device__ __forceinline__ void init(int lane) {
    const int h = lane >> 5, c = lane & 31, i = lane & 15, b16 = (lane >> 4) & 1;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) row_frag[kk] = chunk_off<D>(c, 2 * kk + h);
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int second = 0; second < 2; ++second) {
        const int row = 4 * h + (i >> 2) + 8 * second;
        const int chunk = 4 * db + 2 * b16 + ((i & 3) >> 1);
        trans[db][second] = chunk_off<D>(row, chunk) + (i & 1) * 8;
      }
  }
};
// transposed A operand for rows 16 cc + {4h.., 8 + 4h..} of a stage, column block db
template <int D>
__device__ __forceinline__ bf16x8 read_trans(const char* stage, const FragOffsets<D>& fo, int cc,
                                             int db) {
  bf16x4 lo = lds_read_tr(stage + fo.trans[db][0] + cc * 16 * D * 2);
  bf16x4 hi = lds_read_tr(stage + fo.trans[db][1] + cc * 16 * D * 2);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  Decode the id so
// that all units of one head land on the same XCDs and share its K/V (or Q/dO) lines in L2.
__device__ __forceinline__ void decode_block(int bid, int Hq, int& unit, int& head) {
  constexpr int kXcds = 8;
  const int xcd = bid % kXcds, local = bid / kXcds;
  if (kXcds % Hq == 0) {
    const int per = kXcds / Hq;          // XCDs per head
    head = xcd % Hq;
    unit = local * per + xcd / Hq;
  } else if (Hq % kXcds == 0) {
    const int per = Hq / kXcds;          // heads per XCD
    head = xcd + kXcds * (local % per);
    unit = local / per;
  } else {
    unit = bid / Hq;
    head = bid % Hq;
  }
}
inline unsigned grid_for(int units, int Hq) { return (unsigned)(((long long)units * Hq + 7) / 8 * 8); }

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
constexpr int kTargetUnits = 2048;
constexpr int kNoSplitSteps = 1 << 28;
constexpr long long kSortAboveSteps = 1024;  // (tile step, head) pairs; below: sweep order

struct PlanArgs {
  const int32_t* cu;
  int B, N, Hq, g, shift, no_split;
  int force_ch[2];  // > 0: chunk length given by the caller (tuning), per direction
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
  if (sorted) {
    hist[0][tid] = hist[1][tid] = 0;
    cursor[0][tid] = cursor[1][tid] = 0;
  }
  __syncthreads();

  // mode 0: count unit costs (sorted plans only); mode 1: write units.
  int mode = sorted ? 0 : 1;
#pragma unroll 1
  for (;;) {
    // Every (document, tile) once.  All waves walk all batches of 64 documents; tile 0 of a
    // document is taken by one lane of the wave that owns the batch, and the further tiles of
    // longer documents are swept by whole waves, the long documents dealt round-robin to the
    // waves.  One call site for the per-tile code.
    int long_rank = 0;
#pragma unroll 1
    for (int b0 = 0; b0 < a.B; b0 += 64) {
      const int b = b0 + lane;
      int s = 0, e = 0;
      if (b < a.B) { s = cu[b]; e = cu[b + 1]; }
      const int T = (e - s + kTile - 1) / kTile;
      unsigned long long pending = __ballot(T > 1);
      const bool own_batch = ((b0 >> 6) % (kPlanThreads / 64)) == wave;
      int ss = s, ee = e, i = 0, TT = own_batch ? min(T, 1) : 0;
#pragma unroll 1
      for (;;) {
#pragma unroll 1
        while (__any(i < TT)) {
          if (i < TT) {
            const int row0 = ss + i * kTile;
#pragma unroll 1
            for (int d = 0; d < 2; ++d) {
              const int n = d == 0 ? (min(row0 + kTile, ee) - 1 - ss) / kStep + 1
                                   : (ee - row0 + kStep - 1) / kStep;
              const int nc = (n + ch[d] - 1) / ch[d], base = n / nc, rem = n % nc;
              if (mode == 0) {
                atomicAdd(&hist[d][(base - 1) >> a.shift], nc - rem);
                if (rem) atomicAdd(&hist[d][base >> a.shift], rem);
                if (nc > 1) atomicAdd(&split[d], nc);
              } else {
                int slot0 = -1;
                if (nc > 1 || (d == 1 && a.g > 1)) {
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
          if ((long_rank++ % (kPlanThreads / 64)) == wave) {
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
    // the capacities are worst-case bounds; an overflow cannot happen, but never trust it
    const bool ok = n_units[0] <= a.max_units && n_units[1] <= a.max_units &&
                    n_comb[0] <= a.max_combine && n_comb[1] <= a.max_combine &&
                    n_slots[0] <= a.max_slots[0] && n_slots[1] <= a.max_slots[1];
    hdr->status = VARLEN_ATTN_OK;
    hdr->n_row_units = ok ? n_units[0] : 0;
    hdr->n_col_units = ok ? n_units[1] : 0;
    hdr->n_row_combine = ok ? n_comb[0] : 0;
    hdr->n_col_combine = ok ? n_comb[1] : 0;
    hdr->row_chunk_steps = ch[0];
    hdr->col_chunk_steps = ch[1];
    hdr->n_row_slots = n_slots[0];
    hdr->n_col_slots = n_slots[1];
    hdr->sorted = sorted;
    for (int i = 0; i < 4; ++i) hdr->reserved[i] = 0;
    hdr->pairs = (int64_t)pairs;
  }
}

// ----------------------------------------------------------------------------------------
// Partial results of a cut chain are kept in "fragment layout": the accumulator registers
// exactly as the producing wave holds them, so that every store and load is a contiguous
// 1 KiB per wave: float index (((wave * DB + db) * 4 + rq) * 64 + lane) * 4 + e  for
// accumulator register r = 4 rq + e of column block db.  128 * D floats per tensor.
// ----------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void store_frag(float* base, const f32x16 (&acc)[D / 32], int wave,
                                           int lane) {
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      f32x4 t = {acc[db][4 * rq], acc[db][4 * rq + 1], acc[db][4 * rq + 2], acc[db][4 * rq + 3]};
      *reinterpret_cast<f32x4*>(base + ((((size_t)wave * (D / 32) + db) * 4 + rq) * 64 + lane) * 4) = t;
    }
}
template <int D>
__device__ __forceinline__ f32x4 load_frag4(const float* base, int wave, int lane, int db, int rq) {
  return *reinterpret_cast<const f32x4*>(base + ((((size_t)wave * (D / 32) + db) * 4 + rq) * 64 + lane) * 4);
}
template <int D> constexpr size_t frag_floats() { return (size_t)kTile * D; }
// forward partial: O fragment, then running max m[4][64] and row sum l[4][64]
template <int D> constexpr size_t fwd_partial_floats() { return frag_floats<D>() + 2 * kThreads; }

// bf16 store of one accumulator row set: lane owns row `row`, columns 32 db + 8 rq + 4h + e
template <int D>
__device__ __forceinline__ void store_rows(__bf16* row_ptr, const f32x16 (&acc)[D / 32], int h,
                                           float mul) {
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int d0 = 32 * db + 8 * rq + 4 * h;
      *reinterpret_cast<uint2*>(row_ptr + d0) =
          pack4(acc[db][4 * rq] * mul, acc[db][4 * rq + 1] * mul, acc[db][4 * rq + 2] * mul,
                acc[db][4 * rq + 3] * mul);
    }
}

// ----------------------------------------------------------------------------------------
// Forward.  One workgroup per (row unit, q head); wave w owns query rows row0 + 32w .. +31.
// Computes S^T = K Q^T so that a query is a lane column; online softmax in the exp2 domain
// with a lazily updated running max; O^T += V^T P^T.  A unit that covers its whole chain
// normalises and stores O and LSE; otherwise it stores the unnormalised accumulator with its
// running max and row sum for fwd_combine_kernel.
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads, 2)
fwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
           const varlen_attn_plan_header* __restrict__ hdr,
           const varlen_attn_unit* __restrict__ units, __bf16* __restrict__ o,
           float* __restrict__ lse, float* __restrict__ partials, int N, int Hq, int Hkv,
           float scale, int max_units) {
  constexpr int KK = D / 16, DB = D / 32;
  constexpr int NS = 4;                              // pipeline stages of 32 keys
  constexpr int kStageBytes = kSub * D * 2;
  constexpr int LPS = 2 * StageLoader<D>::kPerWave;  // DMA loads per thread per stage (K and V)
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
  const size_t kv_stride = (size_t)Hkv * D;
  const unsigned lds_k = lds_addr_of(smem), lds_v = lds_k + NS * kStageBytes;

  StageLoader<D> loader;
  loader.init(wave, lane, (unsigned)(kv_stride * 2));
  auto issue = [&](int sub, int stage) {
    const int row0 = kv_begin + kSub * min(sub, n_sub - 1);
    loader.issue(kbase, row0, it.doc_end - 1, lds_k + stage * kStageBytes, wave);
    loader.issue(vbase, row0, it.doc_end - 1, lds_v + stage * kStageBytes, wave);
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
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) s = mfma(lds_read_frag(kt, fo.row_frag[kk]), qf[kk], s);
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
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const bf16x8 pb = pack8(s, 8 * cc);
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma(read_trans<D>(vt, fo, cc, db), pb, oacc[db]);
    }
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
  auto issue = [&](int sub, int stage) {
    const int row0 = kv_begin + kSub * min(sub, n_sub - 1);
    loader.issue(kbase, row0, it.doc_end - 1, lds_k + stage * kStageBytes, wave);
    loader.issue(vbase, row0, it.doc_end - 1, lds_v + stage * kStageBytes, wave);
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
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      s = mfma(lds_read_frag(kt, fo.row_frag[kk]), qf[kk], s);
      dp = mfma(lds_read_frag(vt, fo.row_frag[kk]), dof[kk], dp);
    }
    const bool diag = kv0 + kSub - 1 > wave_row0;
    const int t = my_row - kv0 - 4 * h;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cs, -lse2));
      if (diag && 8 * (r / 4) + (r % 4) > t) p = 0.f;
      s[r] = p * (dp[r] - dsum_row);
    }
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const bf16x8 dsb = pack8(s, 8 * cc);
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(read_trans<D>(kt, fo, cc, db), dsb, acc[db]);
    }
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
// Backward, dK and dV.  One workgroup per (column unit, q head): wave w owns key rows
// row0 + 32w .. +31, keeps their K and V fragments in registers, and sweeps the unit's
// query steps (from the diagonal towards the document end).
//   S = Q K^T, dP = dO V^T (query rows in registers r, key on the lane),
//   dV^T += dO^T P,  dK^T += Q^T dS.
// With grouped-query attention, or when the chain is cut, the unit stores fp32 partials
// [dK | dV] that sum_combine_kernel adds up over the chunks and the q heads of the group.
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads, 1)
bwd_dkv_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
               const __bf16* __restrict__ v, const __bf16* __restrict__ d_o,
               const float* __restrict__ lse2, const float* __restrict__ dsum,
               const varlen_attn_plan_header* __restrict__ hdr,
               const varlen_attn_unit* __restrict__ units, __bf16* __restrict__ dk,
               __bf16* __restrict__ dv, float* __restrict__ partials, int N, int Hq, int Hkv,
               float scale, int max_units) {
  constexpr int KK = D / 16, DB = D / 32;
  // Two stages of kStep = 64 query rows: one stage of lookahead is a whole stage of compute
  // (this kernel runs one workgroup per CU), and 64 KB of tiles keeps every LDS offset inside
  // the 16-bit immediate of the read instructions.
  constexpr int NS = 2;
  constexpr int kStageBytes = kStep * D * 2;
  constexpr int kStatBytes = 512;             // lse2[64] then dsum[64], one copy per wave
  using Loader = StageLoader<D, kStep>;
  constexpr int LPS = 2 * Loader::kPerWave + 2;
  // Q stages | dO stages | per-wave stat copies
  __shared__ __attribute__((aligned(1024))) char smem[2 * NS * kStageBytes + NS * 4 * kStatBytes];

  int unit_idx, head;
  decode_block(blockIdx.x, Hq, unit_idx, head);
  // both loads in flight together; the unit array always has max_units >= grid / Hq entries
  const int n_units = hdr->n_col_units;
  const varlen_attn_unit it = units[min(unit_idx, max_units - 1)];
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
  const unsigned lds_q = lds_addr_of(smem), lds_do = lds_q + NS * kStageBytes;
  const unsigned lds_stat = lds_do + NS * kStageBytes + wave * kStatBytes;
  const char* stat_base = smem + 2 * NS * kStageBytes + wave * kStatBytes;

  Loader loader;
  loader.init(wave, lane, (unsigned)((size_t)Hq * D * 2));
  auto issue = [&](int st, int stage) {
    const int q0 = it.row0 + kStep * (it.step_begin + min(st, n_steps - 1));
    loader.issue(qbase, q0, it.doc_end - 1, lds_q + stage * kStageBytes, wave);
    loader.issue(dobase, q0, it.doc_end - 1, lds_do + stage * kStageBytes, wave);
    dma_floats64(lse_h, q0, it.doc_end - 1, lds_stat + stage * 4 * kStatBytes, lane);
    dma_floats64(dsum_h, q0, it.doc_end - 1, lds_stat + stage * 4 * kStatBytes + 256, lane);
  };
#pragma unroll
  for (int st = 0; st < NS - 1; ++st) issue(st, st);

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
  wait_all_vm_visible();

  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) { dkacc[i] = f32x16(0.f); dvacc[i] = f32x16(0.f); }

  // One 32-query block of a stage against this wave's 32 keys.  MASKED: the block may touch
  // the diagonal or run past the document end (queries there are clamped duplicates).
  auto block = [&](const char* qt, const char* dot, const char* st, int qb, int q0, auto masked_c) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int qb0 = q0 + 32 * qb;
    if (MASKED && (qb0 + 31 < wave_kv0 || qb0 >= it.doc_end)) return;  // wave-uniform
    f32x16 s = f32x16(0.f), dp = f32x16(0.f);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      s = mfma(lds_read_frag(qt, fo.row_frag[kk] + qb * 32 * D * 2), kf[kk], s);
      dp = mfma(lds_read_frag(dot, fo.row_frag[kk] + qb * 32 * D * 2), vf[kk], dp);
    }
    f32x16 p;
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int rel = 32 * qb + 8 * rq + 4 * h;
      const f32x4 l4 = *reinterpret_cast<const f32x4*>(st + rel * 4);
      const f32x4 d4 = *reinterpret_cast<const f32x4*>(st + 256 + rel * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = 4 * rq + e;
        float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cs, -l4[e]));
        if (MASKED) {
          const int t = q0 + rel + e;
          if (t < my_kv || t >= it.doc_end) pv = 0.f;
        }
        p[r] = pv;
        s[r] = pv * (dp[r] - d4[e]);
      }
    }
#pragma unroll
    for (int cc = 0; cc < 2; ++cc) {
      const bf16x8 pb = pack8(p, 8 * cc);
      const bf16x8 dsb = pack8(s, 8 * cc);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        dvacc[db] = mfma(read_trans<D>(dot + qb * 32 * D * 2, fo, cc, db), pb, dvacc[db]);
        dkacc[db] = mfma(read_trans<D>(qt + qb * 32 * D * 2, fo, cc, db), dsb, dkacc[db]);
      }
    }
  };
  // A whole 64-query stage away from the diagonal and the document end: the two 32-query
  // blocks are software-pipelined by hand (this kernel runs one wave per SIMD, so nothing
  // else hides LDS latency or overlaps the exponentials with the matrix pipe):
  //   R0 | M1(0) + R1 | V(0) with M1(1) + T0 | M2(0) with V(1) + T1 | M2(1)
  // R: row-fragment and statistics reads, T: transposed-fragment reads, M1: S and dP,
  // V: P and dS on the vector ALU, M2: dV and dK.  Each matrix instruction is written next to
  // the vector and LDS work that should ride on it, and the fences keep that order.
  auto stage_fast = [&](const char* qt, const char* dot, const char* st) {
    constexpr int EPM = 16 / (2 * KK);  // score elements handled beside each matrix instruction
    bf16x8 qa[KK], da[KK], qb[KK], db_[KK];
    bf16x8 tq0[2][DB], td0[2][DB], tq1[2][DB], td1[2][DB];
    f32x4 l0[4], d0[4], l1[4], d1[4];
    // softmax of element r of one block: p = 2^(s cs - lse2), ds = p (dp - D)
    auto soft = [&](f32x16& sv, const f32x16& dpv, f32x16& pv, const f32x4* l, const f32x4* dd, int r) {
      const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], cs, -l[r >> 2][r & 3]));
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
      for (int e = 0; e < EPM; ++e) soft(s0, dp0, p0, l0, d0, EPM * 2 * kk + e);
      td0[kk / DB][kk % DB] = read_trans<D>(dot, fo, kk / DB, kk % DB);
      __builtin_amdgcn_sched_barrier(0);
      dp1 = mfma(db_[kk], vf[kk], dp1);
#pragma unroll
      for (int e = 0; e < EPM; ++e) soft(s0, dp0, p0, l0, d0, EPM * (2 * kk + 1) + e);
      tq0[kk / DB][kk % DB] = read_trans<D>(qt, fo, kk / DB, kk % DB);
      if ((kk + 1) * 2 * EPM % 8 == 0) {
        constexpr int i = (kk + 1) * 2 * EPM / 8 - 1;
        pb0[i] = pack8(p0, 8 * i);
        dsb0[i] = pack8(s0, 8 * i);
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
      for (int e = 0; e < EPM; ++e) soft(s1, dp1, p1, l1, d1, EPM * 2 * j + e);
      td1[j / DB][j % DB] = read_trans<D>(dot + 32 * D * 2, fo, j / DB, j % DB);
      __builtin_amdgcn_sched_barrier(0);
      dkacc[j % DB] = mfma(tq0[j / DB][j % DB], dsb0[j / DB], dkacc[j % DB]);
#pragma unroll
      for (int e = 0; e < EPM; ++e) soft(s1, dp1, p1, l1, d1, EPM * (2 * j + 1) + e);
      tq1[j / DB][j % DB] = read_trans<D>(qt + 32 * D * 2, fo, j / DB, j % DB);
      if ((j + 1) * 2 * EPM % 8 == 0) {
        constexpr int i = (j + 1) * 2 * EPM / 8 - 1;
        pb1[i] = pack8(p1, 8 * i);
        dsb1[i] = pack8(s1, 8 * i);
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
    if (!wave_active) return;
    const int step = it.step_begin + st;
    const int q0 = it.row0 + kStep * step;
    const char* qt = smem + ST * kStageBytes;
    const char* dot = smem + (NS + ST) * kStageBytes;
    const char* stt = stat_base + ST * 4 * kStatBytes;
    if (step < 2 || q0 + kStep > it.doc_end) {
      block(qt, dot, stt, 0, q0, std::true_type{});
      block(qt, dot, stt, 1, q0, std::true_type{});
    } else {
      stage_fast(qt, dot, stt);
    }
  };
  for (int st = 0; st < n_steps; st += NS) {
    body(st, std::integral_constant<int, 0>{});
    if (st + 1 >= n_steps) break;
    body(st + 1, std::integral_constant<int, 1>{});
  }
  wait_vm<0>();  // nothing may still be landing in LDS when the workgroup retires

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
                                            int Hin, int G, float scale0) {
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
  const int n_parts = it.n_chunks * G;
  auto part = [&](int j) {
    return *reinterpret_cast<const f32x4*>(p0 + ((size_t)(j / G) * Hin + (j % G)) * psize);
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

// One launch for both backward reductions: the first `dkv_blocks` workgroups sum the
// [dK | dV] partials (over chunks and the q heads of a group), the rest sum the dQ partials.
template <int D>
__global__ void __launch_bounds__(kThreads)
bwd_combine_kernel(const varlen_attn_plan_header* __restrict__ hdr,
                   const varlen_attn_combine_item* __restrict__ col_items,
                   const varlen_attn_combine_item* __restrict__ row_items,
                   const float* __restrict__ col_partials, const float* __restrict__ row_partials,
                   __bf16* __restrict__ dk, __bf16* __restrict__ dv, __bf16* __restrict__ dq,
                   int Hq, int Hkv, float scale, int dkv_blocks) {
  if ((int)blockIdx.x < dkv_blocks)
    sum_combine<D, 2>(blockIdx.x, hdr->n_col_combine, col_items, col_partials, dk, dv, Hq, Hq / Hkv, scale);
  else
    sum_combine<D, 1>(blockIdx.x - dkv_blocks, hdr->n_row_combine, row_items, row_partials, dq, nullptr,
                      Hq, 1, scale);
}

// ----------------------------------------------------------------------------------------
// Measurement aid: nothing but bf16 MFMA 32x32x16 on every SIMD (two waves each, four
// independent accumulator chains per wave), operands held in registers.  `random_operands`
// fills A and B with hashed mantissas and signs instead of 1.0: what the matrix pipe sustains
// then is the practical ceiling for kernels whose operands are real data.
// ----------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads, 2)
mfma_rate_kernel(float* __restrict__ out, int iters, int random_operands) {
  bf16x8 a[4], b[4];
  f32x16 c[4];
  unsigned x = (blockIdx.x * kThreads + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    unsigned w[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      x = x * 1664525u + 1013904223u;
      const unsigned y = x ^ (x >> 15);
      // 1.0 with hashed sign and 7-bit mantissa in each half word, or plain 1.0
      w[e] = random_operands ? (0x3f803f80u ^ (y & 0x807f807fu)) : 0x3f803f80u;
    }
    a[u] = __builtin_bit_cast(bf16x8, uint4{w[0], w[1], w[2], w[3]});
    b[u] = __builtin_bit_cast(bf16x8, uint4{w[4], w[5], w[6], w[7]});
    c[u] = f32x16(0.f);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int rep = 0; rep < 4; ++rep)
#pragma unroll
      for (int u = 0; u < 4; ++u) c[u] = mfma(a[u], b[(u + rep) & 3], c[u]);
  }
  float sum = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += c[u][r];
  if (sum == 12345.678f) out[0] = sum;  // keeps the chains alive; practically never true
}

// ----------------------------------------------------------------------------------------
// Optional per-kernel timing (host-side HIP events only; off by default).
// ----------------------------------------------------------------------------------------
enum KernelId { kPlan = 0, kFwd, kFwdCombine, kDq, kDkv, kBwdCombine, kNumKernels };
const char* const kKernelNames[kNumKernels] = {
    "plan_kernel", "fwd_kernel", "fwd_combine_kernel", "bwd_dq_kernel", "bwd_dkv_kernel",
    "bwd_combine_kernel"};
struct Profiler {
  std::mutex mu;
  bool enabled = false;
  struct Rec { int id; hipEvent_t start, stop; };
  std::vector<Rec> recs;
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};
Profiler& profiler() { static Profiler p; return p; }

// Brackets one launch with events when profiling is on.
struct ScopedKernelTimer {
  hipStream_t stream; hipEvent_t stop = nullptr;
  ScopedKernelTimer(int id, hipStream_t s) : stream(s) {
    Profiler& p = profiler();
    if (!p.enabled) return;
    std::lock_guard<std::mutex> g(p.mu);
    hipEvent_t start = p.get();
    stop = p.get();
    if (!start || !stop) { stop = nullptr; return; }
    (void)hipEventRecord(start, stream);
    p.recs.push_back({id, start, stop});
  }
  ~ScopedKernelTimer() { if (stop) (void)hipEventRecord(stop, stream); }
};


inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

bool params_ok(const varlen_attn_params* p) {
  if (!p) return false;
  if (p->total_tokens < 1 || p->num_docs < 1 || p->num_q_heads < 1 || p->num_kv_heads < 1) return false;
  if (p->num_q_heads % p->num_kv_heads) return false;
  if (!(p->softmax_scale > 0.f) || !(p->softmax_scale < 3.0e38f)) return false;
  return true;
}

// Capacities depend on the params only.  Slots: enough for kTargetUnits (unit, head) pairs,
// never more than 8 per tile; with grouped-query attention every column tile takes a slot.
bool layout_of(const varlen_attn_params* p, varlen_attn_workspace_layout* L, int* slots_cap) {
  if (!params_ok(p) || (p->head_dim != 64 && p->head_dim != 128)) return false;
  const long long tiles = (long long)p->total_tokens / kTile + p->num_docs;
  if (tiles > (1 << 24)) return false;
  const int Hq = p->num_q_heads, g = Hq / p->num_kv_heads;
  const long long cap = std::min<long long>((kTargetUnits + Hq - 1) / Hq, 8 * tiles);
  *slots_cap = (int)cap;
  L->max_units = (int)(tiles + cap);
  L->max_combine = (int)tiles;
  L->max_row_slots = (int)cap;
  L->max_col_slots = (int)(cap + (g > 1 ? tiles : 0));
  const size_t frag = (size_t)kTile * p->head_dim * sizeof(float);
  const size_t fwd_part = frag + 2 * kThreads * sizeof(float);
  size_t off = align_up(sizeof(varlen_attn_plan_header), 256);
  L->row_units_offset = off; off = align_up(off + sizeof(varlen_attn_unit) * L->max_units, 256);
  L->col_units_offset = off; off = align_up(off + sizeof(varlen_attn_unit) * L->max_units, 256);
  L->row_combine_offset = off; off = align_up(off + sizeof(varlen_attn_combine_item) * L->max_combine, 256);
  L->col_combine_offset = off; off = align_up(off + sizeof(varlen_attn_combine_item) * L->max_combine, 256);
  // D = rowsum(dO * O) [Hq, N], then LSE * log2(e) [Hq, N]
  L->dsum_offset = off; off = align_up(off + 2 * sizeof(float) * (size_t)Hq * p->total_tokens, 256);
  L->row_partials_offset = off; off = align_up(off + fwd_part * Hq * L->max_row_slots, 256);
  L->col_partials_offset = off; off = align_up(off + 2 * frag * Hq * L->max_col_slots, 256);
  L->total_bytes = off;
  return true;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check_common(const varlen_attn_params* p, const void* const* ptrs, int n_ptrs, void* ws,
                 size_t ws_bytes, varlen_attn_workspace_layout* L, int* slots_cap) {
  if (!params_ok(p)) return VARLEN_ATTN_INVALID_ARG;
  for (int i = 0; i < n_ptrs; ++i)
    if (!ptrs[i]) return VARLEN_ATTN_INVALID_ARG;
  if (!ws) return VARLEN_ATTN_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return VARLEN_ATTN_UNSUPPORTED;
  for (int i = 0; i < n_ptrs; ++i)
    if (!aligned16(ptrs[i])) return VARLEN_ATTN_UNSUPPORTED;
  if (!aligned16(ws)) return VARLEN_ATTN_UNSUPPORTED;
  if (!layout_of(p, L, slots_cap)) return VARLEN_ATTN_UNSUPPORTED;
  if (ws_bytes < L->total_bytes) return VARLEN_ATTN_WORKSPACE_TOO_SMALL;
  return VARLEN_ATTN_OK;
}

struct Regions {
  varlen_attn_plan_header* hdr;
  varlen_attn_unit *row_units, *col_units;
  varlen_attn_combine_item *row_comb, *col_comb;
  float *dsum, *row_part, *col_part;
};
Regions regions_of(char* ws, const varlen_attn_workspace_layout& L) {
  return Regions{reinterpret_cast<varlen_attn_plan_header*>(ws),
                 reinterpret_cast<varlen_attn_unit*>(ws + L.row_units_offset),
                 reinterpret_cast<varlen_attn_unit*>(ws + L.col_units_offset),
                 reinterpret_cast<varlen_attn_combine_item*>(ws + L.row_combine_offset),
                 reinterpret_cast<varlen_attn_combine_item*>(ws + L.col_combine_offset),
                 reinterpret_cast<float*>(ws + L.dsum_offset),
                 reinterpret_cast<float*>(ws + L.row_partials_offset),
                 reinterpret_cast<float*>(ws + L.col_partials_offset)};
}

int launch_plan(const varlen_attn_params* p, const int32_t* cu, const Regions& R,
                const varlen_attn_workspace_layout& L, int slots_cap, hipStream_t stream) {
  int shift = 0;
  const int max_cost = (p->total_tokens + kStep - 1) / kStep;
  while ((max_cost - 1) >> shift >= kPlanBins) ++shift;
  PlanArgs a;
  a.cu = cu; a.B = p->num_docs; a.N = p->total_tokens; a.Hq = p->num_q_heads;
  a.g = p->num_q_heads / p->num_kv_heads; a.shift = shift;
  a.no_split = (p->flags & VARLEN_ATTN_FLAG_NO_SPLIT) ? 1 : 0;
  a.force_ch[0] = (p->flags >> 8) & 0xFF;
  a.force_ch[1] = (p->flags >> 16) & 0xFF;
  a.hdr = R.hdr; a.units[0] = R.row_units; a.units[1] = R.col_units;
  a.comb[0] = R.row_comb; a.comb[1] = R.col_comb;
  a.max_units = L.max_units; a.max_combine = L.max_combine;
  a.max_slots[0] = L.max_row_slots; a.max_slots[1] = L.max_col_slots; a.slots_cap = slots_cap;
  ScopedKernelTimer timer(kPlan, stream);
  plan_kernel<<<1, kPlanThreads, 0, stream>>>(a);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

template <int D>
void launch_fwd(const varlen_attn_params* p, const void* q, const void* k, const void* v, void* o,
                float* lse, const Regions& R, const varlen_attn_workspace_layout& L,
                hipStream_t stream) {
  const int N = p->total_tokens, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  {
    ScopedKernelTimer timer(kFwd, stream);
    fwd_kernel<D><<<dim3(grid_for(L.max_units, Hq)), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, R.hdr, R.row_units, (__bf16*)o, lse,
        R.row_part, N, Hq, Hkv, p->softmax_scale, L.max_units);
  }
  if (!(p->flags & VARLEN_ATTN_FLAG_NO_SPLIT)) {
    ScopedKernelTimer timer(kFwdCombine, stream);
    fwd_combine_kernel<D><<<dim3((unsigned)L.max_combine * Hq * (kTile * D / 4 / kThreads)), kThreads, 0, stream>>>(
        R.hdr, R.row_comb, R.row_part, (__bf16*)o, lse, N, Hq);
  }
}

template <int D>
void launch_bwd(const varlen_attn_params* p, const void* q, const void* k, const void* v,
                const void* o, const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                const Regions& R, const varlen_attn_workspace_layout& L, hipStream_t stream) {
  const int N = p->total_tokens, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  const float scale = p->softmax_scale;
  float* lse2 = R.dsum + (size_t)Hq * N;
  {
    // also writes D = rowsum(dO * O) and LSE * log2(e), which the dK/dV kernel reads
    ScopedKernelTimer timer(kDq, stream);
    bwd_dq_kernel<D><<<dim3(grid_for(L.max_units, Hq)), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)o, (const __bf16*)d_o,
        lse, R.dsum, lse2, R.hdr, R.row_units, (__bf16*)dq, R.row_part, N, Hq, Hkv, scale,
        L.max_units);
  }
  {
    ScopedKernelTimer timer(kDkv, stream);
    bwd_dkv_kernel<D><<<dim3(grid_for(L.max_units, Hq)), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)d_o, lse2, R.dsum, R.hdr,
        R.col_units, (__bf16*)dk, (__bf16*)dv, R.col_part, N, Hq, Hkv, scale, L.max_units);
  }
  const bool split = !(p->flags & VARLEN_ATTN_FLAG_NO_SPLIT);
  if (split || Hq != Hkv) {
    constexpr int kBlocksPerItem = kTile * D / 4 / kThreads;
    const int dkv_blocks = L.max_combine * Hkv * 2 * kBlocksPerItem;
    const int dq_blocks = split ? L.max_combine * Hq * kBlocksPerItem : 0;
    ScopedKernelTimer timer(kBwdCombine, stream);
    bwd_combine_kernel<D><<<dim3((unsigned)(dkv_blocks + dq_blocks)), kThreads, 0, stream>>>(
        R.hdr, R.col_comb, R.row_comb, R.col_part, R.row_part, (__bf16*)dk, (__bf16*)dv, (__bf16*)dq,
        Hq, Hkv, scale, dkv_blocks);
  }
}

}  // namespace

extern "C" {

size_t varlen_attn_workspace_bytes(const varlen_attn_params* params) {
  varlen_attn_workspace_layout L;
  int cap;
  if (!layout_of(params, &L, &cap)) return 0;
  return L.total_bytes;
}

int varlen_attn_workspace_regions(const varlen_attn_params* params,
                                  varlen_attn_workspace_layout* out) {
  if (!out || !params_ok(params)) return VARLEN_ATTN_INVALID_ARG;
  int cap;
  if (!layout_of(params, out, &cap)) return VARLEN_ATTN_UNSUPPORTED;
  return VARLEN_ATTN_OK;
}

int varlen_attn_plan(const varlen_attn_params* params, const int32_t* cu_seqlens, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  varlen_attn_workspace_layout L;
  int cap;
  const void* ptrs[] = {cu_seqlens};
  const int rc = check_common(params, ptrs, 1, workspace, workspace_bytes, &L, &cap);
  if (rc != VARLEN_ATTN_OK) return rc;
  return launch_plan(params, cu_seqlens, regions_of(static_cast<char*>(workspace), L), L, cap,
                     static_cast<hipStream_t>(hip_stream));
}

int varlen_attn_fwd(const varlen_attn_params* params, const void* q, const void* k, const void* v,
                    const int32_t* cu_seqlens, void* o, float* lse, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  varlen_attn_workspace_layout L;
  int cap;
  const void* ptrs[] = {q, k, v, cu_seqlens, o, lse};
  int rc = check_common(params, ptrs, 6, workspace, workspace_bytes, &L, &cap);
  if (rc != VARLEN_ATTN_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const Regions R = regions_of(static_cast<char*>(workspace), L);
  rc = launch_plan(params, cu_seqlens, R, L, cap, stream);
  if (rc != VARLEN_ATTN_OK) return rc;
  if (params->head_dim == 128) launch_fwd<128>(params, q, k, v, o, lse, R, L, stream);
  else launch_fwd<64>(params, q, k, v, o, lse, R, L, stream);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

int varlen_attn_bwd(const varlen_attn_params* params, const void* q, const void* k, const void* v,
                    const void* o, const float* lse, const void* d_o, const int32_t* cu_seqlens,
                    void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  varlen_attn_workspace_layout L;
  int cap;
  const void* ptrs[] = {q, k, v, o, lse, d_o, cu_seqlens, dq, dk, dv};
  int rc = check_common(params, ptrs, 10, workspace, workspace_bytes, &L, &cap);
  if (rc != VARLEN_ATTN_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const Regions R = regions_of(static_cast<char*>(workspace), L);
  if (!(params->flags & VARLEN_ATTN_FLAG_REUSE_PLAN)) {
    rc = launch_plan(params, cu_seqlens, R, L, cap, stream);
    if (rc != VARLEN_ATTN_OK) return rc;
  }
  if (params->head_dim == 128) launch_bwd<128>(params, q, k, v, o, lse, d_o, dq, dk, dv, R, L, stream);
  else launch_bwd<64>(params, q, k, v, o, lse, d_o, dq, dk, dv, R, L, stream);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

int varlen_attn_check(const void* workspace, void* hip_stream) {
  if (!workspace) return VARLEN_ATTN_INVALID_ARG;
  varlen_attn_plan_header hdr;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (hipMemcpyAsync(&hdr, workspace, sizeof(hdr), hipMemcpyDeviceToHost, stream) != hipSuccess)
    return VARLEN_ATTN_LAUNCH_FAILED;
  if (hipStreamSynchronize(stream) != hipSuccess) return VARLEN_ATTN_LAUNCH_FAILED;
  return hdr.status;
}

int varlen_attn_profile(int enable) {
  Profiler& p = profiler();
  std::lock_guard<std::mutex> g(p.mu);
  for (auto& r : p.recs) { p.pool.push_back(r.start); p.pool.push_back(r.stop); }
  p.recs.clear();
  p.enabled = enable != 0;
  return VARLEN_ATTN_OK;
}

int varlen_attn_profile_read(varlen_attn_kernel_time* out, int capacity) {
  if (!out || capacity < 1) return VARLEN_ATTN_INVALID_ARG;
  Profiler& p = profiler();
  std::lock_guard<std::mutex> g(p.mu);
  float total[kNumKernels] = {0};
  int count[kNumKernels] = {0};
  for (auto& r : p.recs) {
    float ms = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
      return VARLEN_ATTN_LAUNCH_FAILED;
    total[r.id] += ms;
    count[r.id] += 1;
    p.pool.push_back(r.start);
    p.pool.push_back(r.stop);
  }
  p.recs.clear();
  int n = 0;
  for (int i = 0; i < kNumKernels && n < capacity; ++i) {
    if (!count[i]) continue;
    out[n].name = kKernelNames[i];
    out[n].launches = count[i];
    out[n].total_ms = total[i];
    ++n;
  }
  return n;
}

int varlen_attn_mfma_rate(int random_operands, int iterations, void* device_scratch,
                          void* hip_stream, float* tflops) {
  if (!device_scratch || !tflops || iterations < 1 || iterations > (1 << 24))
    return VARLEN_ATTN_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return VARLEN_ATTN_LAUNCH_FAILED;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return VARLEN_ATTN_LAUNCH_FAILED;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return VARLEN_ATTN_LAUNCH_FAILED; }
  const unsigned grid = 2u * (unsigned)cus;
  float ms = 0.f;
  bool ok = true;
  for (int pass = 0; pass < 2 && ok; ++pass) {   // the first pass warms the clocks up
    ok = hipEventRecord(e0, stream) == hipSuccess;
    mfma_rate_kernel<<<dim3(grid), kThreads, 0, stream>>>(static_cast<float*>(device_scratch),
                                                          iterations, random_operands);
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, stream) == hipSuccess &&
         hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || ms <= 0.f) return VARLEN_ATTN_LAUNCH_FAILED;
  const double flops = (double)grid * (kThreads / 64) * (double)iterations * 16.0 * 32768.0;
  *tflops = (float)(flops / (ms * 1e-3) / 1e12);
  return VARLEN_ATTN_OK;
}

const char* varlen_attn_status_string(int status) {
  switch (status) {
    case VARLEN_ATTN_OK: return "ok";
    case VARLEN_ATTN_INVALID_ARG: return "invalid argument";
    case VARLEN_ATTN_UNSUPPORTED: return "unsupported head_dim or misaligned pointer";
    case VARLEN_ATTN_WORKSPACE_TOO_SMALL: return "workspace too small";
    case VARLEN_ATTN_LAUNCH_FAILED: return "kernel launch failed";
    case VARLEN_ATTN_BAD_CU_SEQLENS: return "malformed cu_seqlens";
    default: return "unknown status";
  }
}

}  // extern "C"
