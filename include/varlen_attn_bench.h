/*
 * varlen_attn_bench.h - benchmarking aids that are not part of the attention library's ABI.
 *
 * Two groups.  (1) Per-kernel timing of the attention library's own launches with HIP events:
 * exported by libvarlen_attn.so (the launch sites live there) but declared only here, for
 * benchmarks.  (2) Probes of what the matrix pipe and the LDS of the GPU sustain on the
 * instruction mix of the attention kernels: exported by libvarlen_attn_bench.so, which holds
 * nothing else.  Status codes are those of varlen_attn.h.
 */
#ifndef VARLEN_ATTN_BENCH_H_
#define VARLEN_ATTN_BENCH_H_

#include <stddef.h>
#include <stdint.h>

#include "varlen_attn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Optional per-kernel timing for benchmarks.  While enabled (enable != 0), every kernel
 * launch made by this library is bracketed by two HIP events recorded on the launch's own
 * stream (host-side objects; no device memory).  Calling it again, with either value,
 * drops the records collected so far.  Off by default; not thread-safe against concurrent
 * launches that should not be timed. */
typedef struct {
  const char* name; /* static string, e.g. "bwd_dkv_kernel" */
  int32_t launches; /* number of launches recorded */
  float total_ms;   /* sum of their durations */
} varlen_attn_kernel_time;
int varlen_attn_profile(int enable);

/* Waits for the recorded events, writes one entry per kernel that was launched (at most
 * `capacity`), clears the records and returns the number of entries, or a negative status.
 * Blocks the host. */
int varlen_attn_profile_read(varlen_attn_kernel_time* out, int capacity);

/* Measurement aid for benchmarks: runs, on `hip_stream`, a kernel that issues nothing but
 * bf16 MFMA 32x32x16 from registers on every SIMD (2^4 * `iterations` instructions per wave,
 * 8 waves per compute unit), twice, and writes the rate of the second run to the HOST float
 * `tflops`.  random_operands = 0: all operands 1.0; 1: hashed signs and mantissas, which is
 * what the matrix pipe sustains on real data.  `device_scratch`: any 4 writable device
 * bytes (practically never written).  Blocks the host.  Returns VARLEN_ATTN_OK,
 * VARLEN_ATTN_INVALID_ARG or VARLEN_ATTN_LAUNCH_FAILED. */
int varlen_attn_bench_mfma_rate(int random_operands, int iterations, void* device_scratch,
                          void* hip_stream, float* tflops);

/* Measurement aid: the same for the LDS reads of the attention kernels (row fragments with
 * ds_read_b128 when transposed = 0, transposed fragments with ds_read_b64_tr_b16 when 1; 16
 * reads in flight per wave, 8 waves per compute unit): bytes per nominal clock per compute
 * unit, written to the HOST float.  Blocks the host. */
int varlen_attn_bench_lds_rate(int transposed, int iterations, void* device_scratch, void* hip_stream,
                         float* bytes_per_clock_per_cu);

/* Measurement aid: do matrix and vector instructions overlap on one SIMD?  One workgroup of
 * eight waves per compute unit; waves 0-3 (one per SIMD) run work_a, waves 4-7 work_b.  Work per
 * iteration: 0 = sixteen bf16 MFMA 32x32x16 on four accumulators; 1 = sixty-four independent
 * fp32 fma; 2 = sixteen v_exp_f32; 3 = sixteen times (one MFMA, four fma) in one instruction
 * stream; 4 = sixteen times (one MFMA, one exp); -1 = nothing.  Supported pairs: (w, -1) for
 * every w, (0,0), (1,1), (2,2), (3,3), (4,4), (0,1), (0,2).  Runs twice on `hip_stream` and
 * writes the second run's time per iteration, in clocks of the nominal 2.4 GHz, to the HOST
 * float.  `device_scratch`: any 4 writable device bytes.  Blocks the host. */
int varlen_attn_bench_overlap(int work_a, int work_b, int iterations, void* device_scratch,
                              void* hip_stream, float* clocks_per_iteration);

/* Measurement aid: fp32 atomic adds (mode 0) or plain stores (mode 1) in the access pattern of the
 * single-kernel backward: 256 workgroups, each adding a block of 64 rows x 128 floats per stage,
 * `stages` times; the block of workgroup b at stage s is region (b + s * stride) % regions of
 * `device_buffer` (regions * 32 KiB <= buffer_bytes; the buffer's contents are overwritten).
 * Runs twice on `hip_stream` and writes the rate of the second run, in GB/s of 4-byte values, to
 * the HOST float.  Blocks the host. */
int varlen_attn_bench_atomic_rate(int mode, int stages, int regions, int stride, void* device_buffer,
                                  size_t buffer_bytes, void* hip_stream, float* gigabytes_per_second);

/* Measurement aid: copies `bytes` (a multiple of 16; both DEVICE pointers 16-byte aligned) with a
 * plain kernel named bench_copy_kernel, enqueued on `hip_stream`: reads `bytes` and writes `bytes`
 * of HBM, the known quantity that the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 run are
 * scaled by. */
int varlen_attn_bench_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* VARLEN_ATTN_BENCH_H_ */
