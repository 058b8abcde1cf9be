/*
 * moe_shard.h -- C ABI of the MoE Expert-module forward pass on one GPU's shard (gfx950).
 *
 * The operation is the Expert module of an MoE transformer layer as the paper describes it
 * ("MoE Model Architectures": a gating network with Top-K selection dispatches every token to
 * its most relevant expert networks; some models add always-active shared experts), evaluated
 * on the share of the weights one device holds under the paper's Expert-module strategies:
 * tensor parallelism (each device holds a slice of every expert's intermediate dimension;
 * "Tensor Parallelism", and the ILP constraint that the TP degree divides the expert
 * intermediate size) and expert parallelism (each device holds a contiguous subset of experts;
 * "Expert Parallelism", and the constraint that the EP degree divides the expert count).
 * No collective is performed: a TP shard emits the unreduced partial sum, an EP shard receives
 * the whole batch with global routing decisions and emits only its local experts' contribution.
 *
 * Conventions for every entry point
 *   - returns MOE_OK (0) or a negative MOE_ERR_* code; never throws;
 *   - arguments are validated on the host before any HIP call, so invalid arguments return an
 *     error without touching the device;
 *   - never allocates, never synchronises: all work is enqueued on `stream` (a hipStream_t
 *     passed as void*, NULL = the default stream);
 *   - every pointer except `shard` is a DEVICE pointer owned by the caller, who keeps it alive
 *     until the stream has drained; `shard` is a HOST pointer read during the call only;
 *   - bf16 tensors are passed as `const void*` / `void*` (2 bytes per element, row-major);
 *   - data-dependent sizes (rows per expert) stay on the device in `expert_offsets`; buffers
 *     indexed by permuted row are sized by the capacity cap = T*k.
 */
#ifndef MOE_SHARD_H
#define MOE_SHARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MOE_OK = 0,
  MOE_ERR_INVALID_ARG = -1,       /* null pointer, size out of range, non-divisible shard   */
  MOE_ERR_UNSUPPORTED_SHAPE = -2, /* valid in principle, but outside what the kernels handle */
  MOE_ERR_WORKSPACE = -3,         /* workspace smaller than moe_workspace_bytes()            */
  MOE_ERR_HIP = -4                /* a HIP launch reported an error                          */
};

/* flags */
enum {
  MOE_RENORM_TOPK = 1u << 0,  /* moe_route_topk: divide the k gate weights by their sum       */
  MOE_LOGITS_GIVEN = 1u << 1, /* moe_route_topk: `logits` is an input, x / w_router unused    */
  MOE_Y_PERM_BF16 = 1u << 2,  /* moe_expert_ffn / moe_combine: y_perm, y_shared are bf16 (default fp32) */
  MOE_OUT_F32 = 1u << 3,      /* moe_combine: y_out is fp32 (default bf16)                    */
  MOE_FFN_SKIP_GATEUP = 1u << 4, /* moe_expert_ffn: do not run GEMM1; h_workspace is an input  */
  MOE_FFN_SKIP_DOWN = 1u << 5,   /* moe_expert_ffn: stop after GEMM1; y_perm is not written    */
  MOE_FFN_TILED = 1u << 6,       /* moe_expert_ffn: tiled kernels whatever the cost estimate says */
  MOE_FFN_LEAVE_ROOM = 1u << 7   /* moe_expert_ffn: streaming kernels leave 1/16 of the compute units free */
};

/* limits of this implementation */
#define MOE_MAX_EXPERTS 256 /* E      */
#define MOE_MAX_TOPK 16     /* k      */

/*
 * Shard descriptor: which part of the layer's experts this device holds.
 *   n_local_experts = E / E_e, expert_offset = first global expert id held (EP);
 *   inter_slice     = I / E_t, and the weight pointers passed to moe_expert_ffn already are
 *                     that slice: rows [p*I_s,(p+1)*I_s) of gate and up, the same columns of
 *                     down (TP).
 * Valid iff 1 <= n_local_experts, expert_offset >= 0, expert_offset + n_local_experts <=
 * n_experts, n_local_experts divides n_experts, inter_slice divides inter_full.
 */
typedef struct {
  int32_t n_experts;       /* E, global */
  int32_t n_local_experts; /* E_loc     */
  int32_t expert_offset;   /* off       */
  int32_t hidden;          /* H         */
  int32_t inter_full;      /* I         */
  int32_t inter_slice;     /* I_s       */
} moe_shard_t;

/*
 * Gating network + Top-K selection ("MoE Model Architectures").
 *   logits[t,e] = sum_h x[t,h] * w_router[h,e]           (fp32 accumulate)
 *   experts ordered by (logit descending, expert id ascending); the first k are selected and
 *   written in that order; gate weight = softmax over all E logits at the selected experts,
 *   divided by the sum of the k selected weights when MOE_RENORM_TOPK is set.
 * x_bf16   [T,H] bf16        (unused, may be NULL, with MOE_LOGITS_GIVEN)
 * w_router [H,E] fp32        (unused, may be NULL, with MOE_LOGITS_GIVEN)
 * logits   [T,E] fp32        output; input with MOE_LOGITS_GIVEN (finite values required)
 * topk_idx [T,k] int32       global expert ids
 * topk_w   [T,k] fp32
 * Requires 1 <= k <= E <= MOE_MAX_EXPERTS, k <= MOE_MAX_TOPK, H % 8 == 0, T >= 0.
 */
int moe_route_topk(const void* x_bf16, const float* w_router, float* logits,
                   int32_t T, int32_t H, int32_t E, int32_t k, uint32_t flags,
                   int32_t* topk_idx, float* topk_w, void* stream);

/*
 * Token permutation by expert (the "dispatch" of the Top-K mechanism, restricted to the
 * experts this shard holds): a stable counting sort of the local assignments a = t*k + j by
 * expert id.
 * x_bf16         [T,H] bf16      (unused, may be NULL, when x_perm is NULL)
 * topk_idx       [T,k] int32 global expert ids (each in [0,E))
 * x_perm         [T*k,H] bf16  rows [0,R) written (row r = x[row_src[r] / k]); rest untouched.
 *                NULL: only the index arrays are computed, for moe_expert_ffn_gather, which
 *                reads the rows of x in place
 * expert_offsets [E_loc+1] int32  exclusive prefix sum of local rows per expert; last = R
 * row_src        [T*k] int32   assignment id of each permuted row, rows [0,R) written
 * slot_row       [T*k] int32   permuted row of each assignment, -1 if its expert is not local
 * workspace      at least moe_workspace_bytes(T,k,shard) bytes, 256-byte aligned
 * Requires H % 8 == 0, 1 <= k <= MOE_MAX_TOPK, T*k < 2^24.
 */
int moe_permute(const void* x_bf16, const int32_t* topk_idx, int32_t T, int32_t k,
                const moe_shard_t* shard, void* x_perm, int32_t* expert_offsets,
                int32_t* row_src, int32_t* slot_row,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * moe_permute for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus
 * the workspace), same results bit for bit; the per-workgroup expert counts of the large-batch
 * path live in a static device array of the library (MOE_PERMUTE_STATIC_MAX_COUNTS int32 = 1 MiB
 * per GPU, held until the process ends).  The call allocates nothing and frees nothing.
 * Limit: ceil(T*k / 1024) * n_local_experts <= MOE_PERMUTE_STATIC_MAX_COUNTS when T*k > 2048 (smaller
 * batches use no scratch); beyond it the call returns MOE_ERR_WORKSPACE and enqueues nothing.
 * The array's device address is resolved on the first call on each device (a host-side lookup,
 * no stream work): make that first call outside a graph capture.  All calls on one GPU share the
 * array: calls that overlap there (different streams, or graphs replayed concurrently) race and
 * must be serialised by the caller.  Nothing in it has to start at zero, so no clearing is done.
 */
#define MOE_PERMUTE_STATIC_MAX_COUNTS 262144
int moe_permute_static(const void* x_bf16, const int32_t* topk_idx, int32_t T, int32_t k,
                       const moe_shard_t* shard, void* x_perm, int32_t* expert_offsets,
                       int32_t* row_src, int32_t* slot_row, void* stream);

/*
 * Expert networks on the permuted rows (grouped SwiGLU FFN, bf16 MFMA, fp32 accumulate).
 * For the rows r in [expert_offsets[e], expert_offsets[e+1]) of local expert e:
 *   g = x_r Wg_e^T, u = x_r Wu_e^T, h = silu(g) * u (rounded once to bf16), y_r = h Wd_e^T.
 * x_perm         [cap_rows,H] bf16
 * expert_offsets [E_loc+1] int32 (device), non-decreasing, last <= cap_rows
 * w_gate, w_up   [E_loc][I_s][H] bf16   (row = output feature, H contiguous)
 * w_down         [E_loc][H][I_s] bf16   (row = output feature, I_s contiguous)
 * h_workspace    [cap_rows,I_s] bf16    the activated intermediate h (output of GEMM1)
 * workspace      at least moe_ffn_workspace_bytes(cap_rows, shard) bytes, 256-byte aligned
 *                (fp32 partial sums of launches that are cut along K); may be NULL when that is 0
 * y_perm         [cap_rows,H] fp32 (bf16 with MOE_Y_PERM_BF16); rows [0,R) written
 * With inter_slice < inter_full, y_perm is the tensor-parallel partial sum.
 * The shared expert is a second call with n_local_experts = 1, expert_offsets = {0,T},
 * x_perm = x.  Requires H % 64 == 0, I_s % 64 == 0, cap_rows >= 0.
 * MOE_FFN_SKIP_GATEUP / MOE_FFN_SKIP_DOWN run one of the two GEMMs alone (operator-level
 * benchmarking, as the paper's latency model is fitted on measured operator latencies).
 * MOE_FFN_TILED: each GEMM normally picks, from a cost estimate, between a weight-streaming kernel
 * (few rows per expert) and the tiled MFMA kernel; with this flag both run tiled.  It is meant
 * for a call that overlaps a tiled call on another stream (routed experts beside a shared
 * expert with a few dozen rows or more): the streaming kernel's workgroups stay resident on every compute unit
 * for the whole launch, and a tiled workgroup, which needs a compute unit's whole LDS, cannot
 * start beside them, so the two calls would run one after the other.  Same results to rounding
 * order; the workspace size covers either choice.
 * MOE_FFN_LEAVE_ROOM is the milder form for the same situation when the call has too few tiles to
 * stream well on the tiled kernels: a streaming kernel then launches 15 of every 16 workgroups it
 * would, so 16 compute units stay free for the other stream.  Same results, bit for bit.
 */
int moe_expert_ffn(const void* x_perm, const int32_t* expert_offsets, int32_t cap_rows,
                   const moe_shard_t* shard, const void* w_gate, const void* w_up,
                   const void* w_down, void* h_workspace, void* y_perm,
                   void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/*
 * moe_expert_ffn without the permuted copy of the activations: row r of the first GEMM's input is
 * x_bf16[row_src[r] / k] (row_src as moe_permute writes it, k the Top-K width), read where it lies.
 * Saves writing and re-reading x_perm (2 * R * H * 2 bytes per layer); everything else as above.
 * x_bf16 [T,H] bf16, row_src [>= R] int32 (device), 1 <= k <= MOE_MAX_TOPK.
 */
int moe_expert_ffn_gather(const void* x_bf16, const int32_t* row_src, int32_t k,
                          const int32_t* expert_offsets, int32_t cap_rows, const moe_shard_t* shard,
                          const void* w_gate, const void* w_up, const void* w_down, void* h_workspace,
                          void* y_perm, void* workspace, size_t workspace_bytes, uint32_t flags,
                          void* stream);

/*
 * Weighted un-permute / combine of the Top-K expert outputs, plus the shared expert:
 *   y[t,:] = sum_{j : slot_row[t*k+j] >= 0} topk_w[t,j] * y_perm[slot_row[t*k+j],:]
 *            + gate_t * y_shared[t,:]                 (if y_shared != NULL)
 *   gate_t = sigmoid(sum_h x[t,h] * w_shared_gate[h]) (if w_shared_gate != NULL, else 1)
 * Tokens with no local expert get zeros.  Sums are fp32 in slot order; one rounding to bf16.
 * y_perm   [*,H] fp32 (bf16 with MOE_Y_PERM_BF16)
 * y_shared [T,H] same element type as y_perm, or NULL
 * x_bf16   [T,H] bf16 and w_shared_gate [H] fp32: both NULL or both non-NULL
 * y_out    [T,H] bf16 (fp32 with MOE_OUT_F32)
 * Requires H % 8 == 0.
 */
int moe_combine(const void* y_perm, const int32_t* slot_row, const float* topk_w,
                int32_t T, int32_t k, int32_t H, const void* y_shared,
                const void* x_bf16, const float* w_shared_gate, void* y_out,
                uint32_t flags, void* stream);

/* Bytes of scratch moe_permute needs for (T, k, shard); 0 on invalid arguments. */
size_t moe_workspace_bytes(int32_t T, int32_t k, const moe_shard_t* shard);

/* Bytes of scratch moe_expert_ffn needs for (cap_rows, shard); 0 if none (or invalid arguments).
 * It holds the fp32 partial sums of whatever the down projection cuts along K for a routing: a
 * few slices of cap_rows x H floats in the decoding regime (and never less than the tiled kernels
 * would need, so that MOE_FFN_TILED may be set), at most 65536 / ceil(H / 256) rows of H floats in
 * the prefill regime (whatever the capacity). */
size_t moe_ffn_workspace_bytes(int32_t cap_rows, const moe_shard_t* shard);

/* Static, NUL-terminated description of a status code. */
const char* moe_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SHARD_H */
