// Measurement probes for benchmarks (not part of the attention library): what the matrix pipe
// and the LDS of this GPU sustain on the instruction mix of the attention kernels.  Built into
// libvarlen_attn_bench.so; declared in include/varlen_attn_bench.h.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "varlen_attn_bench.h"

#include "tiles.hpp"
#include "staging.hpp"
#include "mfma_rate.hpp"

namespace {
// plain copy of 16-byte words: a kernel of known HBM traffic, against which the FETCH_SIZE and
// WRITE_SIZE counters of a profiler run are scaled
__global__ void __launch_bounds__(256) bench_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}
// fp32 adds in the access pattern of the single-kernel backward: per stage a workgroup adds a
// block of 64 rows x 128 floats (32 KB), wave w columns 32w .. 32w+31, lanes 0-31 one row and
// lanes 32-63 the row four further (an accumulator tile).  mode 0: atomic adds, 1: plain stores.
// The block of workgroup b at stage s is region (b + s * stride) % regions.
__global__ void __launch_bounds__(256) bench_atomic_kernel(float* buf, int stages, int regions, int stride, int mode) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5, c = lane & 31;
  for (int s = 0; s < stages; ++s) {
    const size_t region = (size_t)(((long long)blockIdx.x + (long long)s * stride) % regions);
    float* base = buf + region * 64 * 128 + 32 * wave + c;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float* p = base + (32 * qb + 8 * (r / 4) + 4 * h + r % 4) * 128;
        if (mode == 0) unsafeAtomicAdd(p, 1.0f);
        else *p = 1.0f;
      }
  }
}
// Do matrix and vector instructions overlap on one SIMD?  A workgroup of eight waves: waves
// 0-3 (one per SIMD) run work A, waves 4-7 work B.  Work per iteration: 0 sixteen bf16 MFMA
// 32x32x16 on four accumulators, 1 sixty-four independent fp32 fma, 2 sixteen v_exp_f32,
// 3 sixteen times (MFMA, four fma) in one instruction stream, 4 sixteen times (MFMA, exp),
// -1 nothing.
template <int WHAT>
__device__ __forceinline__ void overlap_work(float* out, int iters, int lane) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(1.0f + 0.001f * lane); b[e] = (__bf16)(0.5f); }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = f32x16(0.f);
  float v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) v[i] = 0.001f * (lane + i);
#pragma unroll 1
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      if (WHAT == 0 || WHAT == 3 || WHAT == 4) acc[j & 3] = mfma(a, b, acc[j & 3]);
      if (WHAT == 1 || WHAT == 3) {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[(4 * j + e) & 15] = __builtin_fmaf(v[(4 * j + e) & 15], v[(4 * j + e) & 15], 0.001f);
      }
      if (WHAT == 2 || WHAT == 4) v[j] = __builtin_amdgcn_exp2f(v[j]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
#pragma unroll
  for (int i = 0; i < 16; ++i) s += v[i];
  if (s == 123.456f) out[0] = s;   // practically never: keeps the work alive
}
template <int A, int B>
__global__ void __launch_bounds__(512) bench_overlap_kernel(float* out, int iters) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (wave < 4) { if constexpr (A >= 0) overlap_work<A>(out, iters, lane); }
  else { if constexpr (B >= 0) overlap_work<B>(out, iters, lane); }
}
template <int A, int B>
void launch_overlap(float* out, int iters, unsigned grid, hipStream_t stream) {
  bench_overlap_kernel<A, B><<<dim3(grid), 512, 0, stream>>>(out, iters);
}
}  // namespace

extern "C" {

int varlen_attn_bench_overlap(int work_a, int work_b, int iterations, void* device_scratch,
                              void* hip_stream, float* clocks_per_iteration) {
  if (!device_scratch || !clocks_per_iteration || iterations < 1 || iterations > (1 << 24))
    return VARLEN_ATTN_INVALID_ARG;
  void (*launch)(float*, int, unsigned, hipStream_t) = nullptr;
  const int key = (work_a + 1) * 8 + (work_b + 1);
  switch (key) {
    case 1 * 8 + 0: launch = launch_overlap<0, -1>; break;
    case 2 * 8 + 0: launch = launch_overlap<1, -1>; break;
    case 3 * 8 + 0: launch = launch_overlap<2, -1>; break;
    case 4 * 8 + 0: launch = launch_overlap<3, -1>; break;
    case 5 * 8 + 0: launch = launch_overlap<4, -1>; break;
    case 1 * 8 + 1: launch = launch_overlap<0, 0>; break;
    case 2 * 8 + 2: launch = launch_overlap<1, 1>; break;
    case 3 * 8 + 3: launch = launch_overlap<2, 2>; break;
    case 1 * 8 + 2: launch = launch_overlap<0, 1>; break;
    case 1 * 8 + 3: launch = launch_overlap<0, 2>; break;
    case 4 * 8 + 4: launch = launch_overlap<3, 3>; break;
    case 5 * 8 + 5: launch = launch_overlap<4, 4>; break;
    default: return VARLEN_ATTN_INVALID_ARG;
  }
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int cus = 0, dev = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
    return VARLEN_ATTN_LAUNCH_FAILED;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return VARLEN_ATTN_LAUNCH_FAILED;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return VARLEN_ATTN_LAUNCH_FAILED; }
  float ms = 0.f;
  bool ok = true;
  for (int pass = 0; pass < 2 && ok; ++pass) {   // the first pass warms up
    ok = hipEventRecord(e0, stream) == hipSuccess;
    launch(static_cast<float*>(device_scratch), iterations, (unsigned)cus, stream);
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, stream) == hipSuccess &&
         hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || ms <= 0.f) return VARLEN_ATTN_LAUNCH_FAILED;
  *clocks_per_iteration = (float)((double)ms * 1e-3 * 2.4e9 / iterations);
  return VARLEN_ATTN_OK;
}

int varlen_attn_bench_atomic_rate(int mode, int stages, int regions, int stride, void* device_buffer,
                                  size_t buffer_bytes, void* hip_stream, float* gigabytes_per_second) {
  if (!device_buffer || !gigabytes_per_second || stages < 1 || stages > (1 << 20) || regions < 1 ||
      stride < 0 || (mode != 0 && mode != 1) || (size_t)regions * 32768 > buffer_bytes)
    return VARLEN_ATTN_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return VARLEN_ATTN_LAUNCH_FAILED;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return VARLEN_ATTN_LAUNCH_FAILED; }
  const unsigned grid = 256;
  float ms = 0.f;
  bool ok = true;
  for (int pass = 0; pass < 2 && ok; ++pass) {   // the first pass warms up
    ok = hipEventRecord(e0, stream) == hipSuccess;
    bench_atomic_kernel<<<dim3(grid), 256, 0, stream>>>(static_cast<float*>(device_buffer), stages, regions,
                                                        stride, mode);
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, stream) == hipSuccess &&
         hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || ms <= 0.f) return VARLEN_ATTN_LAUNCH_FAILED;
  *gigabytes_per_second = (float)((double)grid * stages * 32768.0 / (ms * 1e-3) / 1e9);
  return VARLEN_ATTN_OK;
}

int varlen_attn_bench_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst || bytes < 16 || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15) ||
      (reinterpret_cast<uintptr_t>(dst) & 15))
    return VARLEN_ATTN_INVALID_ARG;
  bench_copy_kernel<<<dim3(2048), 256, 0, static_cast<hipStream_t>(hip_stream)>>>(
      static_cast<const uint4*>(src), static_cast<uint4*>(dst), bytes / 16);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

int varlen_attn_bench_mfma_rate(int random_operands, int iterations, void* device_scratch,
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

int varlen_attn_bench_lds_rate(int transposed, int iterations, void* device_scratch, void* hip_stream,
                         float* bytes_per_clock_per_cu) {
  if (!device_scratch || !bytes_per_clock_per_cu || iterations < 1 || iterations > (1 << 24))
    return VARLEN_ATTN_INVALID_ARG;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  int dev = 0, cus = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) != hipSuccess || khz <= 0)
    return VARLEN_ATTN_LAUNCH_FAILED;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess) return VARLEN_ATTN_LAUNCH_FAILED;
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return VARLEN_ATTN_LAUNCH_FAILED; }
  const unsigned grid = 2u * (unsigned)cus;
  float ms = 0.f;
  bool ok = true;
  for (int pass = 0; pass < 2 && ok; ++pass) {
    ok = hipEventRecord(e0, stream) == hipSuccess;
    lds_rate_kernel<<<dim3(grid), kThreads, 0, stream>>>(static_cast<float*>(device_scratch),
                                                         iterations, transposed);
    ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(e1, stream) == hipSuccess &&
         hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (!ok || ms <= 0.f) return VARLEN_ATTN_LAUNCH_FAILED;
  // 16 fragments of 1 KiB per wave and iteration, 8 waves per CU; clocks at the nominal rate
  const double bytes_per_cu = 8.0 * (double)iterations * 16.0 * 1024.0;
  *bytes_per_clock_per_cu = (float)(bytes_per_cu / (ms * 1e-3 * khz * 1e3));
  return VARLEN_ATTN_OK;
}

}  // extern "C"
