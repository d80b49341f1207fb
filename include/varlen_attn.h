/*
 * varlen_attn.h — C ABI of the MI355X (gfx950) document-masked causal attention library.
 *
 * The operation (Section 5.2, "Micro-Batch Time Prediction"): a packed micro-batch holds
 * documents of lengths l_1..l_k, sum N, concatenated along the token axis; a
 * block-diagonal mask keeps attention inside each document, so the cost follows
 * sum_i l_i^2 (Eq. 1) instead of N^2.  The models are decoder-only, so the mask is causal
 * inside each block: token t of document b attends to keys j with cu[b] <= j <= t.
 *
 *   forward :  S = scale * Q K^T (masked),  LSE = log sum exp S,  P = exp(S - LSE),  O = P V
 *   backward:  D = rowsum(dO * O),  dV = P^T dO,  dP = dO V^T,  dS = P * (dP - D),
 *              dQ = scale * dS K,   dK = scale * dS^T Q      (P recomputed from LSE)
 *
 * Grouped-query attention: q-head h reads kv-head h / (num_q_heads / num_kv_heads);
 * dK and dV are summed over the q-heads of each group.
 *
 * Memory: every pointer below except `params` is a DEVICE pointer owned by the caller,
 * 16-byte aligned.  The library allocates nothing, keeps no state between calls and never
 * synchronises with the host (varlen_attn_check excepted); all work is enqueued on
 * `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).
 *
 * Layouts (row-major, contiguous):
 *   q, o, d_o, dq : bf16 [N, num_q_heads,  head_dim]
 *   k, v, dk, dv  : bf16 [N, num_kv_heads, head_dim]
 *   lse           : fp32 [num_q_heads, N]   natural log of sum_j exp(scale * q.k_j)
 *   cu_seqlens    : int32 [num_docs + 1], cu[0] = 0, cu[num_docs] = N, non-decreasing;
 *                   document b owns tokens cu[b] .. cu[b+1]-1; empty documents are legal.
 * Outputs are fully overwritten.  A malformed cu_seqlens is detected on the device: the
 * plan then holds no work items, no output is written, and varlen_attn_check reports it.
 */
#ifndef VARLEN_ATTN_H_
#define VARLEN_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Geometry of the plan.  Every non-empty document is cut into tiles of
 * VARLEN_ATTN_TILE_ROWS consecutive tokens starting at its first token.  The work of a tile
 * is a chain of steps of VARLEN_ATTN_STEP_ROWS rows each:
 *   row chain (forward, dQ):  key steps 0 .. ceil((last valid row of the tile + 1 - cu[b]) / 64) - 1,
 *                             step s holding keys cu[b] + 64 s .. + 63;
 *   column chain (dK, dV):    query steps 0 .. ceil((cu[b+1] - row0) / 64) - 1,
 *                             step s holding queries row0 + 64 s .. + 63.
 * A long chain is cut into chunks of nearly equal length so that a short microbatch still
 * fills the GPU; each chunk is one work unit, and the partial results of a cut chain are
 * summed afterwards in a fixed order (deterministic). */
#define VARLEN_ATTN_TILE_ROWS 128
#define VARLEN_ATTN_STEP_ROWS 64

/* Status codes (0 = success, negative = error). */
#define VARLEN_ATTN_OK 0
#define VARLEN_ATTN_INVALID_ARG (-1)          /* null pointer, non-positive size, Hq % Hkv != 0, bad scale */
#define VARLEN_ATTN_UNSUPPORTED (-2)          /* head_dim not in {64,128}, misaligned pointer */
#define VARLEN_ATTN_WORKSPACE_TOO_SMALL (-3)
#define VARLEN_ATTN_LAUNCH_FAILED (-4)        /* the HIP runtime refused a launch */
#define VARLEN_ATTN_BAD_CU_SEQLENS (-5)       /* reported by varlen_attn_check only */
#define VARLEN_ATTN_PLAN_OVERFLOW (-6)        /* reported by varlen_attn_check only: the plan needed
                                                 more units, reductions or partial-result slots
                                                 than the workspace holds; no work was planned and
                                                 no output is written */

#define VARLEN_ATTN_STATIC_TOO_LARGE (-7)      /* varlen_attn_fwd_static only: the problem needs more
                                                 than VARLEN_ATTN_STATIC_SCRATCH_BYTES of workspace */

/* Size of the workspace that the library itself holds on every GPU it runs on, for
 * varlen_attn_fwd_static. */
#define VARLEN_ATTN_STATIC_SCRATCH_BYTES (40u << 20)

/* flags */
#define VARLEN_ATTN_FLAG_REUSE_PLAN 1 /* fwd, bwd: the workspace still holds the plan that a
                                         preceding varlen_attn_plan / varlen_attn_fwd call with
                                         the same params (apart from this flag) and cu_seqlens
                                         wrote, e.g. for the other layers of the same
                                         micro-batch; the plan step is then left out */
#define VARLEN_ATTN_FLAG_NO_SPLIT 2   /* never cut a chain: every document is then computed
                                         exactly as if it were alone in the microbatch
                                         (bit-identical results under repacking), at the
                                         price of idle compute units on short microbatches */

#define VARLEN_ATTN_FLAG_FUSED_BWD 16 /* bwd: one kernel for dQ, dK and dV, so that S and dP are
                                         computed once for the whole backward (5 contractions per
                                         (query, key) pair instead of the 7 of the two-kernel
                                         form).  dQ is summed with floating-point atomics into an
                                         fp32 array in the workspace and rounded afterwards: its
                                         bits are NOT reproducible from run to run (dK, dV stay
                                         reproducible).  The flag enlarges the workspace by
                                         4 N Hq d bytes: pass it to varlen_attn_workspace_bytes and
                                         to the forward call as well.  On MI355X this form is the
                                         slower one (the atomic adds bound it) and exists for
                                         comparison. */
#define VARLEN_ATTN_FLAG_PLAN_FIRST 32 /* testing: the plan in a launch of its own in front of the forward
                                         also on small microbatches (by default, with at most 64
                                         documents and 256 tiles, the forward workgroups work out
                                         their own units from cu_seqlens and the plan is made beside
                                         them, inside the forward launch) */
#define VARLEN_ATTN_FLAG_PLAN_LARGE 8 /* testing: plan with the general (16-wave) form of the plan kernel
                                         also where the single-wave form would be taken */

/* Tuning: bits 8..15 of flags = longest chunk of a row chain, bits 16..23 = of a column chain,
 * in steps (0 = chosen by the plan from the microbatch; the plan still lengthens a value
 * whose partial results would not fit the workspace). */
/* Tuning: bits 24..27 of flags = q heads per column unit under grouped-query attention (a
 * divisor of Hq / Hkv; 0 = chosen by the plan: more than 1 only on large microbatches). */
#define VARLEN_ATTN_FLAG_GROUP_HEADS(n) (((n) & 0xF) << 24)
#define VARLEN_ATTN_FLAG_CHUNK_STEPS(row, col) ((((row) & 0xFF) << 8) | (((col) & 0xFF) << 16))

typedef struct {
  int32_t total_tokens;  /* N   >= 1 */
  int32_t num_docs;      /* B   >= 1; cu_seqlens has B + 1 entries */
  int32_t num_q_heads;   /* Hq  >= 1 */
  int32_t num_kv_heads;  /* Hkv >= 1, Hq % Hkv == 0 */
  int32_t head_dim;      /* 64 or 128 */
  float softmax_scale;   /* finite, > 0 (usually 1/sqrt(head_dim)) */
  int32_t flags;         /* VARLEN_ATTN_FLAG_* */
} varlen_attn_params;

/* Work unit of the plan: a chunk [step_begin, step_end) of the chain of one tile.  Units are
 * ordered by non-increasing cost class (cost - 1) >> class_shift of their direction (longest
 * jobs first; 32 classes at most); the order inside a class is not defined. */
typedef struct {
  int32_t row0;       /* first token of the tile */
  int32_t doc_start;  /* cu[b]   */
  int32_t doc_end;    /* cu[b+1] */
  int32_t step_begin; /* first step of the chain this unit covers */
  int32_t step_end;   /* one past its last step */
  int32_t slot;       /* partial-result slot, or -1 when the unit covers the whole chain and
                         writes the final output itself */
  int32_t cost;       /* step_end - step_begin */
  int32_t reserved;
} varlen_attn_unit;

/* A tile whose partial results (slots slot0 .. slot0 + n_chunks - 1) must be summed. */
typedef struct {
  int32_t row0;
  int32_t doc_end;
  int32_t slot0;
  int32_t n_chunks;
} varlen_attn_combine_item;

/* Header at the start of the workspace, written by the plan step. */
typedef struct {
  int32_t status;          /* VARLEN_ATTN_OK, VARLEN_ATTN_BAD_CU_SEQLENS or VARLEN_ATTN_PLAN_OVERFLOW */
  int32_t n_row_units;     /* units of the forward / dQ direction */
  int32_t n_col_units;     /* units of the dK/dV direction */
  int32_t n_row_combine;   /* tiles whose row chain was cut */
  int32_t n_col_combine;   /* tiles whose column chain was cut, or all tiles when Hq > Hkv */
  int32_t row_chunk_steps; /* longest chunk allowed in a row chain */
  int32_t col_chunk_steps; /* longest chunk allowed in a column chain */
  int32_t n_row_slots;
  int32_t n_col_slots;
  int32_t row_class_shift; /* row units are in non-increasing order of (cost - 1) >> row_class_shift */
  int32_t col_heads_per_unit; /* grouped-query attention: q heads of one group that a column
                                 unit sweeps one after the other (a divisor of Hq / Hkv; 1: one
                                 unit per q head) */
  int32_t col_class_shift; /* the same for the column units */
  int32_t reserved[2];
  int64_t pairs;           /* sum_b l_b (l_b + 1) / 2: (query, key) pairs inside the mask */
} varlen_attn_plan_header;

/* Byte offsets and capacities of the regions of the workspace (host function). */
typedef struct {
  size_t row_units_offset;
  size_t col_units_offset;
  size_t row_combine_offset;
  size_t col_combine_offset;
  size_t dsum_offset;         /* fp32 D = rowsum(dO * O) [Hq, N], then LSE * log2(e) [Hq, N] */
  size_t row_partials_offset; /* fp32 partial results of cut row chains */
  size_t col_partials_offset; /* fp32 partial results of cut / grouped column chains */
  size_t dq_accumulator_offset; /* fp32 dQ accumulator [N, Hq, d]; present (non-empty) only with
                                   VARLEN_ATTN_FLAG_FUSED_BWD */
  size_t total_bytes;
  int32_t max_units;          /* capacity of each unit array */
  int32_t max_combine;        /* capacity of each combine array */
  int32_t max_row_slots;
  int32_t max_col_slots;
} varlen_attn_workspace_layout;

/* Bytes the caller must provide (device memory, 16-byte aligned); 0 if params are invalid.
 * The size depends on the params only, never on the contents of cu_seqlens: the plan
 * lengthens its chunks until the partial results fit.  Host function, no device work. */
size_t varlen_attn_workspace_bytes(const varlen_attn_params* params);

/* Fills `out`; returns VARLEN_ATTN_OK or VARLEN_ATTN_INVALID_ARG / UNSUPPORTED (host function). */
int varlen_attn_workspace_regions(const varlen_attn_params* params,
                                  varlen_attn_workspace_layout* out);

/* Plan step alone (it is also the first step of varlen_attn_fwd and of varlen_attn_bwd unless
 * VARLEN_ATTN_FLAG_REUSE_PLAN is set): reads cu_seqlens on the device,
 * validates it, and writes header + items into the workspace.  Integer work only. */
int varlen_attn_plan(const varlen_attn_params* params, const int32_t* cu_seqlens,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* Forward (Section 5.2: the attention term of a packed micro-batch, block-diagonal mask, causal
 * inside a document; cost proportional to sum l_i^2, Eq. 1):
 *   S_tj = scale * q_t . k_j for cu[b] <= j <= t,  lse_t = log sum_j exp S_tj,
 *   o_t = sum_j exp(S_tj - lse_t) v_j.
 * q, k, v, cu_seqlens: device, read only.  o [N, Hq, d] bf16 and lse [Hq, N] fp32: device,
 * fully overwritten.  workspace: device, at least varlen_attn_workspace_bytes(params) bytes,
 * written (plan, partial results); it must stay untouched until a varlen_attn_bwd call with
 * VARLEN_ATTN_FLAG_REUSE_PLAN has been enqueued, if one follows.  Returns a host-checkable status
 * (INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, LAUNCH_FAILED) without touching the device on
 * error; device-detected conditions are read with varlen_attn_check. */
int varlen_attn_fwd(const varlen_attn_params* params, const void* q, const void* k,
                    const void* v, const int32_t* cu_seqlens, void* o, float* lse,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* varlen_attn_fwd for callers that can neither allocate nor provide a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same
 * arguments and results (bit for bit) as varlen_attn_fwd, but the workspace is a fixed array of
 * VARLEN_ATTN_STATIC_SCRATCH_BYTES (40 MiB) of device memory inside the library, one copy per
 * GPU, held until the process ends.  The call allocates and frees nothing (its first call on a
 * device looks the array's address up).  A problem whose forward workspace (plan, D / LSE area
 * and row partial results: about 33 - 35 MiB for 4 q heads at head_dim 128, whatever N) exceeds
 * the array is refused with VARLEN_ATTN_STATIC_TOO_LARGE before any device work.
 * plan_status: optional DEVICE int32 (4-byte aligned), or NULL; the plan step writes its status
 * word there as well (VARLEN_ATTN_OK, _BAD_CU_SEQLENS, _PLAN_OVERFLOW), since the caller has no
 * workspace to pass to varlen_attn_check.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 * streams, two host threads) race; serialise them.  Nothing in the array needs to start at
 * zero: every call rewrites the plan and every partial result it reads.  The plan is not kept
 * for a later varlen_attn_bwd (which plans into its own workspace). */
int varlen_attn_fwd_static(const varlen_attn_params* params, const void* q, const void* k,
                           const void* v, const int32_t* cu_seqlens, void* o, float* lse,
                           int32_t* plan_status, void* hip_stream);

/* Backward of the same operation (the B chunk of the schedule DAG of Section 5.2; its cost is
 * the quadratic term of Eq. 1 as well).  With P_tj = exp(S_tj - lse_t), D_t = sum_c dO_tc O_tc:
 *   dV_j = sum_t P_tj dO_t,  dP_tj = dO_t . v_j,  dS_tj = P_tj (dP_tj - D_t),
 *   dQ_t = scale * sum_j dS_tj k_j,  dK_j = scale * sum_t dS_tj q_t
 * (dK, dV also summed over the q heads of a group).  Reads q, k, v, o, lse (as written by the
 * forward) and d_o; dq [N, Hq, d], dk, dv [N, Hkv, d] bf16 are fully overwritten.  Workspace and
 * status as for varlen_attn_fwd.
 * Deterministic: no atomics on floating-point data, results are bit-reproducible (unless
 * VARLEN_ATTN_FLAG_FUSED_BWD asks for the single-kernel form). */
int varlen_attn_bwd(const varlen_attn_params* params, const void* q, const void* k,
                    const void* v, const void* o, const float* lse, const void* d_o,
                    const int32_t* cu_seqlens, void* dq, void* dk, void* dv, void* workspace,
                    size_t workspace_bytes, void* hip_stream);

/* Synchronises `hip_stream` and returns the status word the last plan step left in the
 * workspace (VARLEN_ATTN_OK, VARLEN_ATTN_BAD_CU_SEQLENS or VARLEN_ATTN_PLAN_OVERFLOW), or
 * VARLEN_ATTN_LAUNCH_FAILED when the copy fails.  `workspace` is the device pointer given to the
 * plan / forward / backward call.  The only call that blocks. */
int varlen_attn_check(const void* workspace, void* hip_stream);

/* Static text for a status code; never NULL. */
const char* varlen_attn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* VARLEN_ATTN_H_ */
