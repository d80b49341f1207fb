// Document-masked causal attention, forward and backward, for packed variable-length
// microbatches on MI355X (gfx950 / CDNA4).  Hand-written HIP; wave64; bf16 MFMA
// (v_mfma_f32_32x32x16_bf16) with fp32 accumulation.
//
// The operation is the quadratic term of the micro-batch time model (Section 5.2, Eq. 1):
// documents of lengths l_1..l_k packed into N tokens, block-diagonal mask, causal inside
// each block.  Only (query tile, key tile) pairs that contain an allowed (t, j) are ever
// visited, so the work follows sum l_i^2, not N^2.
//
// Sources: tiles.hpp (types, MFMA, LDS tile addressing and the register conventions),
// staging.hpp (direct-to-LDS loads), plan.hpp, fragments.hpp (partial-result layout), fwd.hpp,
// bwd.hpp; this file holds the profiler, the host side and the C ABI.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>
#include <utility>
#include <mutex>
#include <vector>

#include "varlen_attn.h"
#include "varlen_attn_bench.h"   // declares the event profiler exported from here

#include "tiles.hpp"
#include "staging.hpp"
#include "plan.hpp"
#include "fragments.hpp"
#include "fwd.hpp"
#include "bwd.hpp"

namespace {

// ----------------------------------------------------------------------------------------
// Optional per-kernel timing (host-side HIP events only; off by default).
// ----------------------------------------------------------------------------------------
enum KernelId { kPlan = 0, kFwd, kFwdCombine, kDq, kDkv, kBwdCombine, kPrep, kFusedBwd, kDqFinish, kNumKernels };
const char* const kKernelNames[kNumKernels] = {
    "plan_kernel", "fwd_kernel", "fwd_combine_kernel", "bwd_dq_kernel", "bwd_dkv_kernel",
    "bwd_combine_kernel", "bwd_prep_kernel", "bwd_fused_kernel", "bwd_dq_finish_kernel"};
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

}  // namespace

// ----------------------------------------------------------------------------------------
// Workspace of varlen_attn_fwd_static: device memory that belongs to the library, so that the
// call needs no workspace from the caller and allocates nothing.  Every GPU this library runs
// on holds its own copy of the array, at its own address, until the process ends.  In host
// code the name below is only a handle for hipGetSymbolAddress: the address that kernels and
// copies use is the one that call returns for the current device, kept in StaticScratch.
// ----------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[VARLEN_ATTN_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
struct StaticScratch {
  std::mutex mu;
  void* ptr[kMaxDevices] = {};
};
// Device address of `scratch` on the current device (looked up once per device).
int static_scratch(void** out) {
  static StaticScratch st;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VARLEN_ATTN_LAUNCH_FAILED;
  std::lock_guard<std::mutex> g(st.mu);
  if (!st.ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return VARLEN_ATTN_LAUNCH_FAILED;
    st.ptr[dev] = p;
  }
  *out = st.ptr[dev];
  return VARLEN_ATTN_OK;
}

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
  // every grid (units x heads, reduction blocks: tiles x heads x 2 tensors x 16) stays below 2^31
  if (tiles * Hq * 48 >= (1ll << 31)) return false;
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
  // fused backward: fp32 dQ accumulator [N, Hq, d]
  L->dq_accumulator_offset = off;
  if (p->flags & VARLEN_ATTN_FLAG_FUSED_BWD)
    off = align_up(off + sizeof(float) * (size_t)p->total_tokens * Hq * p->head_dim, 256);
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
  float *dsum, *row_part, *col_part, *dq_acc;
};
Regions regions_of(char* ws, const varlen_attn_workspace_layout& L) {
  return Regions{reinterpret_cast<varlen_attn_plan_header*>(ws),
                 reinterpret_cast<varlen_attn_unit*>(ws + L.row_units_offset),
                 reinterpret_cast<varlen_attn_unit*>(ws + L.col_units_offset),
                 reinterpret_cast<varlen_attn_combine_item*>(ws + L.row_combine_offset),
                 reinterpret_cast<varlen_attn_combine_item*>(ws + L.col_combine_offset),
                 reinterpret_cast<float*>(ws + L.dsum_offset),
                 reinterpret_cast<float*>(ws + L.row_partials_offset),
                 reinterpret_cast<float*>(ws + L.col_partials_offset),
                 reinterpret_cast<float*>(ws + L.dq_accumulator_offset)};
}

PlanArgs plan_args(const varlen_attn_params* p, const int32_t* cu, const Regions& R,
                   const varlen_attn_workspace_layout& L, int slots_cap, int32_t* status_copy) {
  PlanArgs a;
  a.cu = cu; a.B = p->num_docs; a.N = p->total_tokens; a.Hq = p->num_q_heads;
  a.g = p->num_q_heads / p->num_kv_heads;
  a.no_split = (p->flags & VARLEN_ATTN_FLAG_NO_SPLIT) ? 1 : 0;
  a.force_ch[0] = (p->flags >> 8) & 0xFF;
  a.force_ch[1] = (p->flags >> 16) & 0xFF;
  a.force_hpu = (p->flags >> 24) & 0xF;
  a.hdr = R.hdr; a.units[0] = R.row_units; a.units[1] = R.col_units;
  a.comb[0] = R.row_comb; a.comb[1] = R.col_comb;
  a.max_units = L.max_units; a.max_combine = L.max_combine;
  a.max_slots[0] = L.max_row_slots; a.max_slots[1] = L.max_col_slots; a.slots_cap = slots_cap;
  a.status_copy = status_copy;
  return a;
}

// a microbatch with few documents and tiles is planned by a single wave (lower latency)
inline bool small_plan(const varlen_attn_params* p) {
  const long long tiles = (long long)p->total_tokens / kTile + p->num_docs;
  return !(p->flags & VARLEN_ATTN_FLAG_PLAN_LARGE) && p->num_docs <= 2 * kPlanThreadsSmall &&
         tiles <= 4 * kPlanThreadsSmall;
}
// ... and, smaller still, needs no plan launch in front of the forward: its workgroups work out
// their own units while one of them makes the plan (see fwd_kernel).  They take the units in
// the order (tile, chunk), not longest first, so this is only for microbatches whose units are
// resident all at once: the plan cuts chains to fill the 512 / Hq workgroup slots per head as
// long as the tiles take at most three quarters of them (plan_chunk_steps), i.e. up to
// tiles x Hq <= 768.
inline bool self_planned_forward(const varlen_attn_params* p) {
  const long long tiles = (long long)p->total_tokens / kTile + p->num_docs;
  return small_plan(p) && !(p->flags & VARLEN_ATTN_FLAG_PLAN_FIRST) && p->num_docs <= kSelfPlanDocs &&
         tiles <= kSelfPlanTiles && tiles * p->num_q_heads <= 3 * kResidentGroups / 2;
}

int launch_plan(const varlen_attn_params* p, const int32_t* cu, const Regions& R,
                const varlen_attn_workspace_layout& L, int slots_cap, hipStream_t stream,
                int32_t* status_copy = nullptr) {
  const PlanArgs a = plan_args(p, cu, R, L, slots_cap, status_copy);
  ScopedKernelTimer timer(kPlan, stream);
  if (small_plan(p)) plan_kernel<kPlanThreadsSmall><<<1, kPlanThreadsSmall, 0, stream>>>(a);
  else plan_kernel<kPlanThreadsLarge><<<1, kPlanThreadsLarge, 0, stream>>>(a);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

// self_plan: the forward launch makes the plan itself (no plan launch went before)
template <int D>
void launch_fwd(const varlen_attn_params* p, const void* q, const void* k, const void* v, void* o,
                float* lse, const Regions& R, const varlen_attn_workspace_layout& L,
                hipStream_t stream, const PlanArgs* self_plan = nullptr) {
  const int N = p->total_tokens, Hq = p->num_q_heads, Hkv = p->num_kv_heads;
  {
    ScopedKernelTimer timer(kFwd, stream);
    if (self_plan)
      fwd_kernel<D, true><<<dim3(grid_for(L.max_units, Hq) + 1), kThreads, 0, stream>>>(
          (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, R.hdr, R.row_units, (__bf16*)o, lse,
          R.row_part, N, Hq, Hkv, p->softmax_scale, L.max_units, *self_plan);
    else
      fwd_kernel<D, false><<<dim3(grid_for(L.max_units, Hq)), kThreads, 0, stream>>>(
          (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, R.hdr, R.row_units, (__bf16*)o, lse,
          R.row_part, N, Hq, Hkv, p->softmax_scale, L.max_units, PlanArgs{});
  }
  if (!(p->flags & VARLEN_ATTN_FLAG_NO_SPLIT)) {
    ScopedKernelTimer timer(kFwdCombine, stream);
    const int cut_tiles = std::max(1, std::min(L.max_combine, L.max_row_slots / 2));   // see launch_bwd
    fwd_combine_kernel<D><<<dim3((unsigned)cut_tiles * Hq * (kTile * D / 4 / kThreads)), kThreads, 0, stream>>>(
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
  const bool fused = (p->flags & VARLEN_ATTN_FLAG_FUSED_BWD) != 0;
  if (fused) {
    // D = rowsum(dO * O), LSE * log2(e), and the dQ accumulator cleared
    ScopedKernelTimer timer(kPrep, stream);
    constexpr int kRowsPerBlock = kThreads / (D / 8);
    const long long rows = (long long)N * Hq;
    bwd_prep_kernel<D><<<dim3((unsigned)((rows + kRowsPerBlock - 1) / kRowsPerBlock)), kThreads, 0, stream>>>(
        (const __bf16*)o, (const __bf16*)d_o, lse, R.dsum, lse2, R.dq_acc, N, Hq);
  } else {
    // also writes D = rowsum(dO * O) and LSE * log2(e), which the dK/dV kernel reads
    ScopedKernelTimer timer(kDq, stream);
    bwd_dq_kernel<D><<<dim3(grid_for(L.max_units, Hq)), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)o, (const __bf16*)d_o,
        lse, R.dsum, lse2, R.hdr, R.row_units, (__bf16*)dq, R.row_part, N, Hq, Hkv, scale,
        L.max_units);
  }
  const bool split = !(p->flags & VARLEN_ATTN_FLAG_NO_SPLIT);
  // A cut chain has at least two chunks and all chunks of cut chains fit the slots, so at most
  // max_row_slots / 2 tiles are cut in either direction.
  const int cut_tiles = std::max(1, std::min(L.max_combine, L.max_row_slots / 2));
  const unsigned unit_blocks = grid_for(L.max_units, Hq);
  if (fused) {
    // one kernel for dQ, dK and dV; dQ is summed in fp32 in the workspace and rounded afterwards
    ScopedKernelTimer timer(kFusedBwd, stream);
    bwd_dkv_kernel<D, true><<<dim3(unit_blocks), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)d_o, lse2, R.dsum, R.hdr,
        R.col_units, (__bf16*)dk, (__bf16*)dv, R.col_part, N, Hq, Hkv, scale, L.max_units,
        (int)unit_blocks, R.row_comb, L.max_combine, R.row_part, (__bf16*)dq, R.dq_acc);
  } else {
    // behind its units: one workgroup per (cut tile, q head) that sums the dQ partials
    const unsigned dq_blocks = split ? (unsigned)cut_tiles * Hq : 0u;
    ScopedKernelTimer timer(kDkv, stream);
    bwd_dkv_kernel<D, false><<<dim3(unit_blocks + dq_blocks), kThreads, 0, stream>>>(
        (const __bf16*)q, (const __bf16*)k, (const __bf16*)v, (const __bf16*)d_o, lse2, R.dsum, R.hdr,
        R.col_units, (__bf16*)dk, (__bf16*)dv, R.col_part, N, Hq, Hkv, scale, L.max_units,
        (int)unit_blocks, R.row_comb, L.max_combine, R.row_part, (__bf16*)dq, nullptr);
  }
  if (fused) {
    const long long n8 = (long long)N * Hq * D / 8;
    ScopedKernelTimer timer(kDqFinish, stream);
    bwd_dq_finish_kernel<D><<<dim3((unsigned)((n8 + kThreads - 1) / kThreads)), kThreads, 0, stream>>>(
        R.dq_acc, (__bf16*)dq, n8, scale);
  }
  if (split || Hq != Hkv) {
    constexpr int kBlocksPerItem = kTile * D / 4 / kThreads;
    // grouped-query attention: every tile's [dK | dV] is summed over the group; else cut tiles only
    const int col_items = Hq != Hkv ? L.max_combine : cut_tiles;
    ScopedKernelTimer timer(kBwdCombine, stream);
    bwd_combine_kernel<D><<<dim3((unsigned)(col_items * Hkv * 2 * kBlocksPerItem)), kThreads, 0, stream>>>(
        R.hdr, R.col_comb, R.col_part, (__bf16*)dk, (__bf16*)dv, Hq, Hkv, scale);
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
  PlanArgs self;
  const PlanArgs* self_plan = nullptr;
  if (!(params->flags & VARLEN_ATTN_FLAG_REUSE_PLAN)) {
    if (self_planned_forward(params)) {
      self = plan_args(params, cu_seqlens, R, L, cap, nullptr);
      self_plan = &self;
    } else {
      rc = launch_plan(params, cu_seqlens, R, L, cap, stream);
      if (rc != VARLEN_ATTN_OK) return rc;
    }
  }
  if (params->head_dim == 128) launch_fwd<128>(params, q, k, v, o, lse, R, L, stream, self_plan);
  else launch_fwd<64>(params, q, k, v, o, lse, R, L, stream, self_plan);
  return hipGetLastError() == hipSuccess ? VARLEN_ATTN_OK : VARLEN_ATTN_LAUNCH_FAILED;
}

int varlen_attn_fwd_static(const varlen_attn_params* params, const void* q, const void* k,
                           const void* v, const int32_t* cu_seqlens, void* o, float* lse,
                           int32_t* plan_status, void* hip_stream) {
  varlen_attn_workspace_layout L;
  int cap;
  void* ws = nullptr;
  const void* ptrs[] = {q, k, v, cu_seqlens, o, lse};
  // validate against a workspace of unlimited size first: bad arguments keep their own codes
  if (!params_ok(params)) return VARLEN_ATTN_INVALID_ARG;
  for (const void* ptr : ptrs)
    if (!ptr) return VARLEN_ATTN_INVALID_ARG;
  if (plan_status && (reinterpret_cast<uintptr_t>(plan_status) & 3)) return VARLEN_ATTN_UNSUPPORTED;
  if (params->head_dim != 64 && params->head_dim != 128) return VARLEN_ATTN_UNSUPPORTED;
  for (const void* ptr : ptrs)
    if (!aligned16(ptr)) return VARLEN_ATTN_UNSUPPORTED;
  if (!layout_of(params, &L, &cap)) return VARLEN_ATTN_UNSUPPORTED;
  // the forward touches the workspace up to the end of the row partial results only
  if (L.col_partials_offset > (size_t)VARLEN_ATTN_STATIC_SCRATCH_BYTES) return VARLEN_ATTN_STATIC_TOO_LARGE;
  int rc = static_scratch(&ws);
  if (rc != VARLEN_ATTN_OK) return rc;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const Regions R = regions_of(static_cast<char*>(ws), L);
  PlanArgs self;
  const PlanArgs* self_plan = nullptr;
  if (self_planned_forward(params)) {
    self = plan_args(params, cu_seqlens, R, L, cap, plan_status);
    self_plan = &self;
    rc = VARLEN_ATTN_OK;
  } else {
    rc = launch_plan(params, cu_seqlens, R, L, cap, stream, plan_status);
  }
  if (rc != VARLEN_ATTN_OK) return rc;
  if (params->head_dim == 128) launch_fwd<128>(params, q, k, v, o, lse, R, L, stream, self_plan);
  else launch_fwd<64>(params, q, k, v, o, lse, R, L, stream, self_plan);
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

const char* varlen_attn_status_string(int status) {
  switch (status) {
    case VARLEN_ATTN_OK: return "ok";
    case VARLEN_ATTN_INVALID_ARG: return "invalid argument";
    case VARLEN_ATTN_UNSUPPORTED: return "unsupported head_dim or misaligned pointer";
    case VARLEN_ATTN_WORKSPACE_TOO_SMALL: return "workspace too small";
    case VARLEN_ATTN_LAUNCH_FAILED: return "kernel launch failed";
    case VARLEN_ATTN_BAD_CU_SEQLENS: return "malformed cu_seqlens";
    case VARLEN_ATTN_PLAN_OVERFLOW: return "plan does not fit the workspace";
    case VARLEN_ATTN_STATIC_TOO_LARGE: return "problem exceeds the library's static workspace";
    default: return "unknown status";
  }
}

}  // extern "C"
