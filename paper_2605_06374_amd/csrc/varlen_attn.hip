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
constexpr int kKvStep = 64;                   // key rows staged per iteration (fwd, dQ)
constexpr int kQStep = 64;                    // query rows staged per iteration (dK/dV)
constexpr int kThreads = 256;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kRescaleTau = 8.0f;  // running max may lag by up to 2^8 before O is rescaled

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

// A operand = transpose of rows [row_base + 4h + {0..3}] and [row_base + 8 + 4h + {0..3}]
// of a tile, columns 32 * dblk + c.
template <int D>
__device__ __forceinline__ bf16x8 lds_read_trans_frag(const char* tile, int row_base, int dblk,
                                                      int lane) {
  const int i = lane & 15, b16 = (lane >> 4) & 1, h = lane >> 5;
  const int row = row_base + 4 * h + (i >> 2);
  const int chunk = 4 * dblk + 2 * b16 + ((i & 3) >> 1);
  const int sub = (i & 1) * 8;
  bf16x4 lo = lds_read_tr(tile + chunk_off<D>(row, chunk) + sub);
  bf16x4 hi = lds_read_tr(tile + chunk_off<D>(row + 8, chunk) + sub);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
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

// Stage `ROWS` rows x D columns (row stride `stride` elements) into registers, zero beyond
// `row_limit`; then write them, swizzled, into an LDS tile.
template <int D, int ROWS>
struct TileStager {
  static constexpr int kChunks = ROWS * (D / 8) / kThreads;
  uint4 reg[kChunks];
  __device__ __forceinline__ void load(const __bf16* base, size_t stride, int row0, int row_limit,
                                       int tid) {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int id = tid + i * kThreads;
      const int row = id / (D / 8), c = id % (D / 8);
      const int grow = row0 + row;
      reg[i] = uint4{0, 0, 0, 0};
      if (grow < row_limit)
        reg[i] = *reinterpret_cast<const uint4*>(base + (size_t)grow * stride + c * 8);
    }
  }
  __device__ __forceinline__ void store(char* tile, int tid) const {
#pragma unroll
    for (int i = 0; i < kChunks; ++i) {
      const int id = tid + i * kThreads;
      const int row = id / (D / 8), c = id % (D / 8);
      *reinterpret_cast<uint4*>(tile + chunk_off<D>(row, c)) = reg[i];
    }
  }
};

// ----------------------------------------------------------------------------------------
// Plan: cu_seqlens -> validated, cost-ordered tile list (integer work only).
// One workgroup of 1024 threads.  Items are placed by a counting sort on cost, descending
// (longest job first); the order among items of equal cost is not defined.
// ----------------------------------------------------------------------------------------
constexpr int kPlanThreads = 1024;
constexpr int kPlanBins = 1024;

// Visit every (document, tile) pair once: lanes own documents for the first kLaneTiles tiles,
// then whole waves sweep the remaining tiles of long documents.
template <typename F>
__device__ __forceinline__ void for_each_tile(const int32_t* cu, int B, F f) {
  constexpr int kLaneTiles = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = kPlanThreads / 64;
  for (int b0 = wave * 64; b0 < B; b0 += nwaves * 64) {
    const int b = b0 + lane;
    int s = 0, e = 0;
    if (b < B) { s = cu[b]; e = cu[b + 1]; }
    const int T = (e - s + kTile - 1) / kTile;
    for (int i = 0; i < kLaneTiles && i < T; ++i) f(s, e, i);
    unsigned long long longdocs = __ballot(T > kLaneTiles);
    while (longdocs) {
      const int src = __ffsll((long long)longdocs) - 1;
      longdocs &= longdocs - 1;
      const int ss = __shfl(s, src), ee = __shfl(e, src), TT = __shfl(T, src);
      for (int i = kLaneTiles + lane; i < TT; i += 64) f(ss, ee, i);
    }
  }
}

__global__ void __launch_bounds__(kPlanThreads) plan_kernel(const int32_t* __restrict__ cu, int B,
                                                            int N, int shift,
                                                            varlen_attn_plan_header* hdr,
                                                            varlen_attn_item* items,
                                                            int max_items) {
  __shared__ int bad;
  __shared__ int hist[kPlanBins];    // tiles per cost bucket, then start offsets (descending)
  __shared__ int cursor[kPlanBins];
  __shared__ unsigned long long pairs;
  const int tid = threadIdx.x;
  if (tid == 0) { bad = (cu[0] != 0) || (cu[B] != N); pairs = 0; }
  hist[tid] = 0;
  cursor[tid] = 0;
  __syncthreads();
  unsigned long long my_pairs = 0;
  int my_bad = 0;
  for (int b = tid; b < B; b += kPlanThreads) {
    const long long l = (long long)cu[b + 1] - cu[b];
    if (l < 0) my_bad = 1;
    my_pairs += (unsigned long long)(l * (l + 1) / 2);
  }
  if (my_bad) bad = 1;
  __syncthreads();
  if (bad) {
    if (tid == 0) {
      hdr->n_items = 0; hdr->status = VARLEN_ATTN_BAD_CU_SEQLENS; hdr->pairs = 0;
      hdr->max_items = max_items; hdr->reserved[0] = hdr->reserved[1] = hdr->reserved[2] = 0;
    }
    return;
  }
  if (my_pairs) atomicAdd(&pairs, my_pairs);
  for_each_tile(cu, B, [&](int, int, int i) { atomicAdd(&hist[i >> shift], 1); });
  __syncthreads();
  // start[k] = number of tiles in buckets above k  (exclusive suffix sum, Hillis-Steele)
  int v = hist[tid];
  const int own = v;
  for (int off = 1; off < kPlanBins; off <<= 1) {
    const int other = (tid + off < kPlanBins) ? hist[tid + off] : 0;
    __syncthreads();
    v += other;
    hist[tid] = v;
    __syncthreads();
  }
  const int total = hist[0];
  __syncthreads();
  hist[tid] = v - own;
  __syncthreads();
  for_each_tile(cu, B, [&](int s, int e, int i) {
    const int k = i >> shift;
    const int pos = hist[k] + atomicAdd(&cursor[k], 1);
    if (pos < max_items) items[pos] = varlen_attn_item{s + i * kTile, s, e, i + 1};
  });
  if (tid == 0) {
    hdr->n_items = total < max_items ? total : max_items; hdr->status = VARLEN_ATTN_OK;
    hdr->pairs = (int64_t)pairs; hdr->max_items = max_items;
    hdr->reserved[0] = hdr->reserved[1] = hdr->reserved[2] = 0;
  }
}

// ----------------------------------------------------------------------------------------
// Forward.  One workgroup per (item, q head); wave w owns query rows row0 + 32w .. +31.
// Computes S^T = K Q^T so that a query is a lane column; online softmax in the exp2 domain
// with a lazily updated running max; O^T += V^T P^T.
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads, 2)
fwd_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k, const __bf16* __restrict__ v,
           const varlen_attn_plan_header* __restrict__ hdr,
           const varlen_attn_item* __restrict__ items, __bf16* __restrict__ o,
           float* __restrict__ lse, int N, int Hq, int Hkv, float scale) {
  constexpr int KK = D / 16, DB = D / 32;
  constexpr int kTileBytes = kKvStep * D * 2;
  __shared__ __attribute__((aligned(16))) char smem[4 * kTileBytes];  // K0 K1 V0 V1

  const int item_idx = blockIdx.x / Hq, head = blockIdx.x % Hq;
  if (item_idx >= hdr->n_items) return;
  const varlen_attn_item it = items[item_idx];
  const int kvh = head / (Hq / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, c = lane & 31;
  const float cs = scale * kLog2e;

  const int wave_row0 = it.row0 + 32 * wave;
  const int my_row = wave_row0 + c;
  const bool row_valid = my_row < it.doc_end;
  const bool wave_active = wave_row0 < it.doc_end;
  const int wave_last_row = min(wave_row0 + 31, it.doc_end - 1);
  const int wg_last_row = min(it.row0 + kTile, it.doc_end) - 1;
  const int n_steps = (wg_last_row - it.doc_start) / kKvStep + 1;

  bf16x8 qf[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 t = {0, 0, 0, 0};
    if (row_valid)
      t = *reinterpret_cast<const uint4*>(q + ((size_t)my_row * Hq + head) * D + 16 * kk + 8 * h);
    qf[kk] = __builtin_bit_cast(bf16x8, t);
  }

  const __bf16* kbase = k + (size_t)kvh * D;
  const __bf16* vbase = v + (size_t)kvh * D;
  const size_t kv_stride = (size_t)Hkv * D;

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) oacc[i] = f32x16(0.f);
  float m_run = -INFINITY, l_run = 0.f;

  TileStager<D, kKvStep> ks, vs;
  ks.load(kbase, kv_stride, it.doc_start, it.doc_end, tid);
  vs.load(vbase, kv_stride, it.doc_start, it.doc_end, tid);
  ks.store(smem, tid);
  vs.store(smem + 2 * kTileBytes, tid);
  __syncthreads();

  for (int step = 0; step < n_steps; ++step) {
    const int cur = step & 1;
    const int kv0 = it.doc_start + step * kKvStep;
    const char* kt = smem + cur * kTileBytes;
    const char* vt = smem + (2 + cur) * kTileBytes;
    const bool more = step + 1 < n_steps;
    if (more) {
      ks.load(kbase, kv_stride, kv0 + kKvStep, it.doc_end, tid);
      vs.load(vbase, kv_stride, kv0 + kKvStep, it.doc_end, tid);
    }
    if (wave_active && kv0 <= wave_last_row) {
      f32x16 s[2];
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        s[blk] = f32x16(0.f);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          bf16x8 a = lds_read_frag(kt, chunk_off<D>(32 * blk + c, 2 * kk + h));
          s[blk] = mfma(a, qf[kk], s[blk]);
        }
      }
      if (kv0 + kKvStep - 1 > wave_row0) {  // tile touches the diagonal for some row
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = kv0 + 32 * blk + 8 * (r / 4) + 4 * h + (r % 4);
            if (j > my_row) s[blk][r] = -INFINITY;
          }
      }
      float mx = s[0][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = __builtin_fmaxf(mx, s[0][r]);
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = __builtin_fmaxf(mx, s[1][r]);
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
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[blk][r], cs, -m_run));
          s[blk][r] = p;
          psum += p;
        }
      l_run += psum;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
          const bf16x8 pb = pack8(s[blk], 8 * cc);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 a = lds_read_trans_frag<D>(vt, 32 * blk + 16 * cc, db, lane);
            oacc[db] = mfma(a, pb, oacc[db]);
          }
        }
    }
    if (more) {
      ks.store(smem + (cur ^ 1) * kTileBytes, tid);
      vs.store(smem + (2 + (cur ^ 1)) * kTileBytes, tid);
    }
    __syncthreads();
  }

  if (!wave_active) return;
  const float l_tot = half_sum(l_run);
  if (row_valid) {
    const float inv = 1.0f / l_tot;
    __bf16* orow = o + ((size_t)my_row * Hq + head) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int d0 = 32 * db + 8 * rq + 4 * h;
        *reinterpret_cast<uint2*>(orow + d0) =
            pack4(oacc[db][4 * rq] * inv, oacc[db][4 * rq + 1] * inv, oacc[db][4 * rq + 2] * inv,
                  oacc[db][4 * rq + 3] * inv);
      }
    if (h == 0) lse[(size_t)head * N + my_row] = (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}

// ----------------------------------------------------------------------------------------
// Backward, step 0: D[h][t] = sum_c dO[t,h,c] * O[t,h,c]   (fp32)
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads)
rowdot_kernel(const __bf16* __restrict__ o, const __bf16* __restrict__ d_o, float* __restrict__ dsum,
              int N, int Hq) {
  constexpr int LPR = D / 8;  // lanes per row
  const long long row = (long long)blockIdx.x * (kThreads / LPR) + threadIdx.x / LPR;
  const int part = threadIdx.x % LPR;
  float acc = 0.f;
  if (row < (long long)N * Hq) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(o + (size_t)row * D + part * 8);
    const bf16x8 b = *reinterpret_cast<const bf16x8*>(d_o + (size_t)row * D + part * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += (float)a[e] * (float)b[e];
  }
#pragma unroll
  for (int off = LPR / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if (part == 0 && row < (long long)N * Hq) {
    const int t = (int)(row / Hq), hh = (int)(row % Hq);
    dsum[(size_t)hh * N + t] = acc;
  }
}

// ----------------------------------------------------------------------------------------
// Backward, dQ.  Same decomposition as the forward: one workgroup per (item, q head), key
// tiles up to the diagonal.  S^T = K Q^T, dP^T = V dO^T, dS^T = P^T (dP^T - D),
// dQ^T += K^T dS^T.
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads, 2)
bwd_dq_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
              const __bf16* __restrict__ v, const __bf16* __restrict__ d_o,
              const float* __restrict__ lse, const float* __restrict__ dsum,
              const varlen_attn_plan_header* __restrict__ hdr,
              const varlen_attn_item* __restrict__ items, __bf16* __restrict__ dq, int N, int Hq,
              int Hkv, float scale) {
  constexpr int KK = D / 16, DB = D / 32;
  constexpr int kTileBytes = kKvStep * D * 2;
  __shared__ __attribute__((aligned(16))) char smem[4 * kTileBytes];  // K0 K1 V0 V1

  const int item_idx = blockIdx.x / Hq, head = blockIdx.x % Hq;
  if (item_idx >= hdr->n_items) return;
  const varlen_attn_item it = items[item_idx];
  const int kvh = head / (Hq / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, c = lane & 31;
  const float cs = scale * kLog2e;

  const int wave_row0 = it.row0 + 32 * wave;
  const int my_row = wave_row0 + c;
  const bool row_valid = my_row < it.doc_end;
  const bool wave_active = wave_row0 < it.doc_end;
  const int wave_last_row = min(wave_row0 + 31, it.doc_end - 1);
  const int wg_last_row = min(it.row0 + kTile, it.doc_end) - 1;
  const int n_steps = (wg_last_row - it.doc_start) / kKvStep + 1;

  bf16x8 qf[KK], dof[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) {
    uint4 t = {0, 0, 0, 0}, u = {0, 0, 0, 0};
    if (row_valid) {
      const size_t off = ((size_t)my_row * Hq + head) * D + 16 * kk + 8 * h;
      t = *reinterpret_cast<const uint4*>(q + off);
      u = *reinterpret_cast<const uint4*>(d_o + off);
    }
    qf[kk] = __builtin_bit_cast(bf16x8, t);
    dof[kk] = __builtin_bit_cast(bf16x8, u);
  }
  // rows past the document end get LSE = +huge so that their P is exactly 0
  const float lse2 = row_valid ? lse[(size_t)head * N + my_row] * kLog2e : 1e30f;
  const float dsum_row = row_valid ? dsum[(size_t)head * N + my_row] : 0.f;

  const __bf16* kbase = k + (size_t)kvh * D;
  const __bf16* vbase = v + (size_t)kvh * D;
  const size_t kv_stride = (size_t)Hkv * D;

  f32x16 acc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) acc[i] = f32x16(0.f);

  TileStager<D, kKvStep> ks, vs;
  ks.load(kbase, kv_stride, it.doc_start, it.doc_end, tid);
  vs.load(vbase, kv_stride, it.doc_start, it.doc_end, tid);
  ks.store(smem, tid);
  vs.store(smem + 2 * kTileBytes, tid);
  __syncthreads();

  for (int step = 0; step < n_steps; ++step) {
    const int cur = step & 1;
    const int kv0 = it.doc_start + step * kKvStep;
    const char* kt = smem + cur * kTileBytes;
    const char* vt = smem + (2 + cur) * kTileBytes;
    const bool more = step + 1 < n_steps;
    if (more) {
      ks.load(kbase, kv_stride, kv0 + kKvStep, it.doc_end, tid);
      vs.load(vbase, kv_stride, kv0 + kKvStep, it.doc_end, tid);
    }
    if (wave_active && kv0 <= wave_last_row) {
      const bool diag = kv0 + kKvStep - 1 > wave_row0;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        if (kv0 + 32 * blk > wave_last_row) continue;  // wave-uniform
        f32x16 s = f32x16(0.f), dp = f32x16(0.f);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          bf16x8 a = lds_read_frag(kt, chunk_off<D>(32 * blk + c, 2 * kk + h));
          s = mfma(a, qf[kk], s);
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          bf16x8 a = lds_read_frag(vt, chunk_off<D>(32 * blk + c, 2 * kk + h));
          dp = mfma(a, dof[kk], dp);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cs, -lse2));
          if (diag) {
            const int j = kv0 + 32 * blk + 8 * (r / 4) + 4 * h + (r % 4);
            if (j > my_row) p = 0.f;
          }
          s[r] = p * (dp[r] - dsum_row);
        }
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
          const bf16x8 dsb = pack8(s, 8 * cc);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            bf16x8 a = lds_read_trans_frag<D>(kt, 32 * blk + 16 * cc, db, lane);
            acc[db] = mfma(a, dsb, acc[db]);
          }
        }
      }
    }
    if (more) {
      ks.store(smem + (cur ^ 1) * kTileBytes, tid);
      vs.store(smem + (2 + (cur ^ 1)) * kTileBytes, tid);
    }
    __syncthreads();
  }

  if (row_valid) {
    __bf16* row = dq + ((size_t)my_row * Hq + head) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int d0 = 32 * db + 8 * rq + 4 * h;
        *reinterpret_cast<uint2*>(row + d0) =
            pack4(acc[db][4 * rq] * scale, acc[db][4 * rq + 1] * scale,
                  acc[db][4 * rq + 2] * scale, acc[db][4 * rq + 3] * scale);
      }
  }
}

// ----------------------------------------------------------------------------------------
// Backward, dK and dV.  One workgroup per (mirrored item, kv head): item (doc, tile i) of a
// document with T tiles handles key tile T-1-i, whose cost (q tiles at or after it) is i+1,
// so the plan's longest-first order carries over.  Wave w owns key rows kv_row0 + 32w..+31,
// keeps their K and V fragments in registers, and sweeps the q heads of the group and the
// query rows from the diagonal to the document end.
//   S = Q K^T, dP = dO V^T (query rows in registers r, key on the lane),
//   dV^T += dO^T P,  dK^T += Q^T dS.
// ----------------------------------------------------------------------------------------
template <int D>
__global__ void __launch_bounds__(kThreads, 1)
bwd_dkv_kernel(const __bf16* __restrict__ q, const __bf16* __restrict__ k,
               const __bf16* __restrict__ v, const __bf16* __restrict__ d_o,
               const float* __restrict__ lse, const float* __restrict__ dsum,
               const varlen_attn_plan_header* __restrict__ hdr,
               const varlen_attn_item* __restrict__ items, __bf16* __restrict__ dk,
               __bf16* __restrict__ dv, int N, int Hq, int Hkv, float scale) {
  constexpr int KK = D / 16, DB = D / 32;
  constexpr int kTileBytes = kQStep * D * 2;
  // Q0 Q1 dO0 dO1 tiles, then lse2[2][kQStep], dsum[2][kQStep]
  __shared__ __attribute__((aligned(16))) char smem[4 * kTileBytes + 4 * kQStep * 4];
  float* stat = reinterpret_cast<float*>(smem + 4 * kTileBytes);

  const int item_idx = blockIdx.x / Hkv, kvh = blockIdx.x % Hkv;
  if (item_idx >= hdr->n_items) return;
  const varlen_attn_item it = items[item_idx];
  const int g = Hq / Hkv;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, c = lane & 31;
  const float cs = scale * kLog2e;

  const int n_tiles = (it.doc_end - it.doc_start + kTile - 1) / kTile;
  const int kv_row0 = it.doc_start + (n_tiles - it.cost) * kTile;
  const int wave_kv0 = kv_row0 + 32 * wave;
  const int my_kv = wave_kv0 + c;
  const bool kv_valid = my_kv < it.doc_end;
  const bool wave_active = wave_kv0 < it.doc_end;

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

  f32x16 dkacc[DB], dvacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i) { dkacc[i] = f32x16(0.f); dvacc[i] = f32x16(0.f); }

  const int q_steps = (it.doc_end - kv_row0 + kQStep - 1) / kQStep;  // per head
  const int n_steps = q_steps * g;
  const size_t q_stride = (size_t)Hq * D;

  TileStager<D, kQStep> qs, dos;
  float stat_reg = 0.f;
  auto stage_load = [&](int step) {
    const int head = kvh * g + step / q_steps;
    const int q0 = kv_row0 + (step % q_steps) * kQStep;
    qs.load(q + (size_t)head * D, q_stride, q0, it.doc_end, tid);
    dos.load(d_o + (size_t)head * D, q_stride, q0, it.doc_end, tid);
    if (tid < 2 * kQStep) {
      const int t = q0 + (tid % kQStep);
      if (tid < kQStep) stat_reg = t < it.doc_end ? lse[(size_t)head * N + t] * kLog2e : 1e30f;
      else stat_reg = t < it.doc_end ? dsum[(size_t)head * N + t] : 0.f;
    }
  };
  auto stage_store = [&](int buf) {
    qs.store(smem + buf * kTileBytes, tid);
    dos.store(smem + (2 + buf) * kTileBytes, tid);
    if (tid < 2 * kQStep) stat[(tid / kQStep) * 2 * kQStep + buf * kQStep + (tid % kQStep)] = stat_reg;
  };
  stage_load(0);
  stage_store(0);
  __syncthreads();

  for (int step = 0; step < n_steps; ++step) {
    const int cur = step & 1;
    const int q0 = kv_row0 + (step % q_steps) * kQStep;
    const char* qt = smem + cur * kTileBytes;
    const char* dot = smem + (2 + cur) * kTileBytes;
    const float* lse_t = stat + cur * kQStep;
    const float* ds_t = stat + 2 * kQStep + cur * kQStep;
    const bool more = step + 1 < n_steps;
    if (more) stage_load(step + 1);
    if (wave_active) {
#pragma unroll
      for (int qb = 0; qb < kQStep / 32; ++qb) {
        const int qb0 = q0 + 32 * qb;
        // wave-uniform: block wholly above the diagonal for this wave, or past the document
        if (qb0 + 31 < wave_kv0 || qb0 >= it.doc_end) continue;
        f32x16 s = f32x16(0.f), dp = f32x16(0.f);
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          bf16x8 a = lds_read_frag(qt, chunk_off<D>(32 * qb + c, 2 * kk + h));
          s = mfma(a, kf[kk], s);
        }
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          bf16x8 a = lds_read_frag(dot, chunk_off<D>(32 * qb + c, 2 * kk + h));
          dp = mfma(a, vf[kk], dp);
        }
        const bool diag = qb0 < wave_kv0 + 31;
        f32x16 p;
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int rel = 32 * qb + 8 * rq + 4 * h;
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(lse_t + rel);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(ds_t + rel);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * rq + e;
            float pv = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], cs, -l4[e]));
            if (diag && (q0 + rel + e) < my_kv) pv = 0.f;
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
            bf16x8 a = lds_read_trans_frag<D>(dot, 32 * qb + 16 * cc, db, lane);
            dvacc[db] = mfma(a, pb, dvacc[db]);
            bf16x8 a2 = lds_read_trans_frag<D>(qt, 32 * qb + 16 * cc, db, lane);
            dkacc[db] = mfma(a2, dsb, dkacc[db]);
          }
        }
      }
    }
    if (more) stage_store(cur ^ 1);
    __syncthreads();
  }

  if (kv_valid) {
    __bf16* krow = dk + ((size_t)my_kv * Hkv + kvh) * D;
    __bf16* vrow = dv + ((size_t)my_kv * Hkv + kvh) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int d0 = 32 * db + 8 * rq + 4 * h;
        *reinterpret_cast<uint2*>(krow + d0) =
            pack4(dkacc[db][4 * rq] * scale, dkacc[db][4 * rq + 1] * scale,
                  dkacc[db][4 * rq + 2] * scale, dkacc[db][4 * rq + 3] * scale);
        *reinterpret_cast<uint2*>(vrow + d0) =
            pack4(dvacc[db][4 * rq], dvacc[db][4 * rq + 1], dvacc[db][4 * rq + 2],
                  dvacc[db][4 * rq + 3]);
      }
  }
}

// ----------------------------------------------------------------------------------------
// Host side
// ----------------------------------------------------------------------------------------

// ----------------------------------------------------------------------------------------
// Optional per-kernel timing (host-side HIP events only; off by default).
// ----------------------------------------------------------------------------------------
enum KernelId { kPlan = 0, kFwd, kRowdot, kDkv, kDq, kNumKernels };
const char* const kKernelNames[kNumKernels] = {"plan_kernel", "fwd_kernel", "rowdot_kernel",
                                               "bwd_dkv_kernel", "bwd_dq_kernel"};
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

struct Layout {
  int max_items;
  size_t items_off, dsum_off, total;
};

bool params_ok(const varlen_attn_params* p) {
  if (!p) return false;
  if (p->total_tokens < 1 || p->num_docs < 1 || p->num_q_heads < 1 || p->num_kv_heads < 1) return false;
  if (p->num_q_heads % p->num_kv_heads) return false;
  if (!(p->softmax_scale > 0.f) || !(p->softmax_scale < 3.0e38f)) return false;
  return true;
}

bool layout_of(const varlen_attn_params* p, Layout* L) {
  if (!params_ok(p)) return false;
  const long long mi = (long long)p->total_tokens / kTile + p->num_docs;
  if (mi > 0x7fffffffLL / 64) return false;
  L->max_items = (int)mi;
  L->items_off = align_up(sizeof(varlen_attn_plan_header), 256);
  L->dsum_off = align_up(L->items_off + sizeof(varlen_attn_item) * (size_t)mi, 256);
  L->total = align_up(L->dsum_off + sizeof(float) * (size_t)p->num_q_heads * p->total_tokens, 256);
  return true;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check_common(const varlen_attn_params* p, const void* const* ptrs, int n_ptrs, void* ws,
                 size_t ws_bytes, Layout* L) {
  if (!params_ok(p)) return VARLEN_ATTN_INVALID_ARG;
  for (int i = 0; i < n_ptrs; ++i)
    if (!ptrs[i]) return VARLEN_ATTN_INVALID_ARG;
  if (!ws) return VARLEN_ATTN_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return VARLEN_ATTN_UNSUPPORTED;
  for (int i = 0; i < n_ptrs; ++i)
    if (!aligned16(ptrs[i])) return VARLEN_ATTN_UNSUPPORTED;
  if (!aligned16(ws)) return VARLEN_ATTN_UNSUPPORTED;
  if (!layout_of(p, L)) return VARLEN_ATTN_UNSUPPORTED;
  if (ws_bytes < L->total) return VARLEN_ATTN_WORKSPACE_TOO_SMALL;
  return VARLEN_ATTN_OK;
}

int launch_plan(const varlen_attn_params* p, const int32_t* cu, char* ws, const Layout& L,
                hipStream_t stream) {
  int shift = 0;
  const int max_cost = (p->total_tokens + kTile - 1) / kTile;
  while ((max_cost - 1) >> shift >= kPlanBins) ++shift;
  ScopedKernelTimer timer(kPlan, stream);
  plan_kernel<<<1, kPlanThreads, 0, stream>>>(
      cu, p->num_docs, p->total_tokens, shift, reinterpret_cast<varlen_attn_plan_header*>(ws),
      reinterpret_cast<varlen_attn_item*>(ws + L.items_off), L.max_items);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

template <int D>
void launch_bwd(const varlen_attn_params* p, const void* q, const void* k, const void* v,
                const void* o, const float* lse, const void* d_o, void* dq, void* dk, void* dv,
                const varlen_attn_plan_header* hdr, const varlen_attn_item* items, float* dsum,
                const Layout& L, hipStream_t stream) {
  const int N = p->total_tokens, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  const float scale = p->softmax_scale;
  const long long rows = (long long)N * Hq;
  constexpr int kRowsPerBlock = kThreads / (D / 8);
  {
    ScopedKernelTimer timer(kRowdot, stream);
    rowdot_kernel<D><<<(unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock), kThreads, 0, stream>>>(
        (const __bf16*)o, (const __bf16*)d_o, dsum, N, Hq);
  }
  {
    ScopedKernelTimer timer(kDkv, stream);
    bwd_dkv_kernel<D><<<dim3((unsigned)L.max_items * Hkv), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)d_o, lse, dsum, hdr,
        items, (__bf16*)dk, (__bf16*)dv, N, Hq, Hkv, scale);
  }
  {
    ScopedKernelTimer timer(kDq, stream);
    bwd_dq_kernel<D><<<dim3((unsigned)L.max_items * Hq), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)d_o, lse, dsum, hdr,
        items, (__bf16*)dq, N, Hq, Hkv, scale);
  }
}

}  // namespace

extern "C" {

size_t varlen_attn_workspace_bytes(const varlen_attn_params* params) {
  Layout L;
  if (!params_ok(params) || (params->head_dim != 64 && params->head_dim != 128)) return 0;
  if (!layout_of(params, &L)) return 0;
  return L.total;
}

size_t varlen_attn_workspace_items_offset(const varlen_attn_params* params) {
  Layout L;
  if (!layout_of(params, &L)) return 0;
  return L.items_off;
}

int varlen_attn_plan(const varlen_attn_params* params, const int32_t* cu_seqlens, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
  Layout L;
  const void* ptrs[] = {cu_seqlens};
  const int rc = check_common(params, ptrs, 1, workspace, workspace_bytes, &L);
  if (rc != VARLEN_ATTN_OK) return rc;
  return launch_plan(params, cu_seqlens, static_cast<char*>(workspace), L,
                     static_cast<hipStream_t>(hip_stream));
}

int varlen_attn_fwd(const varlen_attn_params* params, const void* q, const void* k, const void* v,
                    const int32_t* cu_seqlens, void* o, float* lse, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
  Layout L;
  const void* ptrs[] = {q, k, v, cu_seqlens, o, lse};
  int rc = check_common(params, ptrs, 6, workspace, workspace_bytes, &L);
  if (rc != VARLEN_ATTN_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  rc = launch_plan(params, cu_seqlens, ws, L, stream);
  if (rc != VARLEN_ATTN_OK) return rc;
  const auto* hdr = reinterpret_cast<const varlen_attn_plan_header*>(ws);
  const auto* items = reinterpret_cast<const varlen_attn_item*>(ws + L.items_off);
  const int N = params->total_tokens, Hq = params->num_q_heads, Hkv = params->num_kv_heads;
  const dim3 grid((unsigned)L.max_items * Hq);
  ScopedKernelTimer timer(kFwd, stream);
  if (params->head_dim == 128)
    fwd_kernel<128><<<grid, kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, hdr, items, (__bf16*)o, lse, N, Hq,
        Hkv, params->softmax_scale);
  else
    fwd_kernel<64><<<grid, kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, hdr, items, (__bf16*)o, lse, N, Hq,
        Hkv, params->softmax_scale);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

int varlen_attn_bwd(const varlen_attn_params* params, const void* q, const void* k, const void* v,
                    const void* o, const float* lse, const void* d_o, const int32_t* cu_seqlens,
                    void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
  Layout L;
  const void* ptrs[] = {q, k, v, o, lse, d_o, cu_seqlens, dq, dk, dv};
  int rc = check_common(params, ptrs, 10, workspace, workspace_bytes, &L);
  if (rc != VARLEN_ATTN_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  char* ws = static_cast<char*>(workspace);
  if (!(params->flags & VARLEN_ATTN_FLAG_REUSE_PLAN)) {
    rc = launch_plan(params, cu_seqlens, ws, L, stream);
    if (rc != VARLEN_ATTN_OK) return rc;
  }
  const auto* hdr = reinterpret_cast<const varlen_attn_plan_header*>(ws);
  const auto* items = reinterpret_cast<const varlen_attn_item*>(ws + L.items_off);
  float* dsum = reinterpret_cast<float*>(ws + L.dsum_off);
  if (params->head_dim == 128)
    launch_bwd<128>(params, q, k, v, o, lse, d_o, dq, dk, dv, hdr, items, dsum, L, stream);
  else
    launch_bwd<64>(params, q, k, v, o, lse, d_o, dq, dk, dv, hdr, items, dsum, L, stream);
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
