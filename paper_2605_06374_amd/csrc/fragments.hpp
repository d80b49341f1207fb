// Fragment layout of fp32 partial results and bf16 row stores.
#ifndef VARLEN_ATTN_FRAGMENTS_HPP_
#define VARLEN_ATTN_FRAGMENTS_HPP_

#include "tiles.hpp"

namespace {

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

}  // namespace

#endif  // VARLEN_ATTN_FRAGMENTS_HPP_
