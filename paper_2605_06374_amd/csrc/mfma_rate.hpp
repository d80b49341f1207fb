// Measurement aids: a kernel of nothing but bf16 MFMA, and one of nothing but LDS fragment reads.
#ifndef VARLEN_ATTN_MFMA_RATE_HPP_
#define VARLEN_ATTN_MFMA_RATE_HPP_

#include "staging.hpp"
#include "tiles.hpp"

namespace {

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
// Measurement aid: nothing but the LDS reads of the attention kernels, from a swizzled 64-row
// tile, 16 independent reads in flight per wave: row fragments (ds_read_b128, transposed = 0) or
// transposed fragments (ds_read_b64_tr_b16 pairs, transposed = 1).  Four waves per workgroup,
// `waves_per_simd` workgroups per CU.
// ----------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads, 2)
lds_rate_kernel(float* __restrict__ out, int iters, int transposed) {
  constexpr int D = 128;
  __shared__ __attribute__((aligned(1024))) char tile[4 * 32 * D * 2];
  for (int i = threadIdx.x; i < (int)sizeof(tile) / 4; i += kThreads)
    reinterpret_cast<unsigned*>(tile)[i] = 0x3f803f80u;
  __syncthreads();
  FragOffsets<D> fo;
  fo.init(threadIdx.x & 63);
  float sum = 0.f;
  for (int it = 0; it < iters; ++it) {
    const char* t = tile + (it & 3) * 32 * D * 2;
    bf16x8 f[16];
    if (transposed) {
#pragma unroll
      for (int j = 0; j < 16; ++j) f[j] = read_trans<D>(t, fo, (j >> 2) & 1, j & 3);
    } else {
#pragma unroll
      for (int j = 0; j < 16; ++j) f[j] = lds_read_frag(t, fo.row_frag[j & 7] + ((j >> 3) & 1) * 16 * D * 2);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) asm volatile("" ::"v"(f[j]));
  }
  if (iters < 0) out[0] = sum;
}

}  // namespace

#endif  // VARLEN_ATTN_MFMA_RATE_HPP_
