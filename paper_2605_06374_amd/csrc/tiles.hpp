// Vector types, constants, MFMA wrapper and swizzled LDS tile addressing shared by every kernel.
//
// Register/lane conventions used by every kernel (L = lane, h = L / 32, c = L % 32):
//   MFMA 32x32x16:  A[i][k]: lane holds i = c, k = 8h + e (e = 0..7)
//                   B[k][j]: lane holds j = c, k = 8h + e
//                   C[i][j]: lane holds j = c, i = 8 (r / 4) + 4h + r % 4 (r = 0..15)
// The kernels always put the softmax row index on the lane (j = c) so that row statistics
// are per-lane scalars, and feed the exponentiated scores straight back as a B operand:
// registers 8cc..8cc+7 of a C tile are the k positions of the cc-th 16-deep slice, standing
// for rows 16cc + 4h + {0..3} and 16cc + 8 + 4h + {0..3}.  The matching A operand is a
// transposed read of a row-major LDS tile (ds_read_b64_tr_b16, twice).
#ifndef VARLEN_ATTN_TILES_HPP_
#define VARLEN_ATTN_TILES_HPP_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

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

}  // namespace

#endif  // VARLEN_ATTN_TILES_HPP_
