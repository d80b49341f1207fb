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
}  // namespace

extern "C" {

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
