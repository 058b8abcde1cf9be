// extern "C" boundary of libmoe_shard: argument validation on the host, then kernel launches.
// Nothing here allocates or synchronises; every error is a return code.
#include "moe_internal.hpp"

namespace moe {
// Rows an expert-parallel shard expects out of a capacity of T*k: its share of the experts.
int expected_rows(int cap_rows, const moe_shard_t* s) {
  const int64_t est = (int64_t)cap_rows * s->n_local_experts / s->n_experts;
  return est < 1 ? (cap_rows > 0 ? 1 : 0) : (int)est;
}
}  // namespace moe

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int shard_status(const moe_shard_t* s) {
  if (s == nullptr) return MOE_ERR_INVALID_ARG;
  if (s->n_experts < 1 || s->n_experts > MOE_MAX_EXPERTS) return MOE_ERR_INVALID_ARG;
  if (s->n_local_experts < 1 || s->expert_offset < 0) return MOE_ERR_INVALID_ARG;
  if ((int64_t)s->expert_offset + s->n_local_experts > s->n_experts) return MOE_ERR_INVALID_ARG;
  if (s->n_experts % s->n_local_experts != 0) return MOE_ERR_INVALID_ARG;  // EP degree must divide E
  if (s->hidden < 1 || s->inter_full < 1 || s->inter_slice < 1) return MOE_ERR_INVALID_ARG;
  if (s->inter_slice > s->inter_full || s->inter_full % s->inter_slice != 0) return MOE_ERR_INVALID_ARG;  // TP degree must divide I
  return MOE_OK;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_HIP; }


}  // namespace

extern "C" {

int moe_route_topk(const void* x_bf16, const float* w_router, float* logits, int32_t T, int32_t H, int32_t E,
                   int32_t k, uint32_t flags, int32_t* topk_idx, float* topk_w, void* stream) {
  if (T < 0 || E < 1 || E > MOE_MAX_EXPERTS || k < 1 || k > E || k > MOE_MAX_TOPK) return MOE_ERR_INVALID_ARG;
  if (flags & ~(uint32_t)(MOE_RENORM_TOPK | MOE_LOGITS_GIVEN)) return MOE_ERR_INVALID_ARG;
  if (logits == nullptr || topk_idx == nullptr || topk_w == nullptr) return MOE_ERR_INVALID_ARG;
  if (!(flags & MOE_LOGITS_GIVEN)) {
    if (x_bf16 == nullptr || w_router == nullptr || H < 8) return MOE_ERR_INVALID_ARG;
    if (H % 8 != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
    if (!aligned16(x_bf16)) return MOE_ERR_INVALID_ARG;
  }
  return hip_status(moe::launch_route_topk(x_bf16, w_router, logits, T, H, E, k, flags, topk_idx, topk_w,
                                           static_cast<hipStream_t>(stream)));
}

size_t moe_workspace_bytes(int32_t T, int32_t k, const moe_shard_t* shard) {
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || shard_status(shard) != MOE_OK) return 0;
  return moe::permute_workspace_bytes(T, k, shard->n_local_experts);
}

size_t moe_ffn_workspace_bytes(int32_t cap_rows, const moe_shard_t* shard) {
  if (cap_rows < 0 || shard_status(shard) != MOE_OK) return 0;
  return moe::ffn_workspace_bytes(cap_rows, moe::expected_rows(cap_rows, shard), shard->n_local_experts, shard->hidden,
                                  shard->inter_slice);
}

int moe_permute(const void* x_bf16, const int32_t* topk_idx, int32_t T, int32_t k, const moe_shard_t* shard,
                void* x_perm, int32_t* expert_offsets, int32_t* row_src, int32_t* slot_row, void* workspace,
                size_t workspace_bytes, void* stream) {
  const int st = shard_status(shard);
  if (st != MOE_OK) return st;
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || k > shard->n_experts) return MOE_ERR_INVALID_ARG;
  if ((int64_t)T * k >= (1 << 24)) return MOE_ERR_INVALID_ARG;
  if (topk_idx == nullptr || expert_offsets == nullptr || row_src == nullptr || slot_row == nullptr)
    return MOE_ERR_INVALID_ARG;
  if (x_perm != nullptr && x_bf16 == nullptr) return MOE_ERR_INVALID_ARG;  // x is read only to fill x_perm
  if (shard->hidden % 8 != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (!aligned16(x_bf16) || !aligned16(x_perm)) return MOE_ERR_INVALID_ARG;
  if (workspace == nullptr || workspace_bytes < moe_workspace_bytes(T, k, shard)) return MOE_ERR_WORKSPACE;
  return hip_status(moe::launch_permute(x_bf16, topk_idx, T, k, shard->hidden, shard->n_local_experts,
                                        shard->expert_offset, x_perm, expert_offsets, row_src, slot_row, workspace,
                                        static_cast<hipStream_t>(stream)));
}

int moe_permute_static(const void* x_bf16, const int32_t* topk_idx, int32_t T, int32_t k, const moe_shard_t* shard,
                       void* x_perm, int32_t* expert_offsets, int32_t* row_src, int32_t* slot_row, void* stream) {
  const int st = shard_status(shard);
  if (st != MOE_OK) return st;
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || k > shard->n_experts) return MOE_ERR_INVALID_ARG;
  if ((int64_t)T * k >= (1 << 24)) return MOE_ERR_INVALID_ARG;
  if (topk_idx == nullptr || expert_offsets == nullptr || row_src == nullptr || slot_row == nullptr)
    return MOE_ERR_INVALID_ARG;
  if (x_perm != nullptr && x_bf16 == nullptr) return MOE_ERR_INVALID_ARG;
  if (shard->hidden % 8 != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (!aligned16(x_bf16) || !aligned16(x_perm)) return MOE_ERR_INVALID_ARG;
  if (moe::permute_static_counts(T, k, shard->n_local_experts) > MOE_PERMUTE_STATIC_MAX_COUNTS)
    return MOE_ERR_WORKSPACE;  // beyond the static scratch: use moe_permute with a caller workspace
  return hip_status(moe::launch_permute_static(x_bf16, topk_idx, T, k, shard->hidden, shard->n_local_experts,
                                               shard->expert_offset, x_perm, expert_offsets, row_src, slot_row,
                                               static_cast<hipStream_t>(stream)));
}

static int expert_ffn_common(const void* x, moe::RowMap rows, const int32_t* expert_offsets, int32_t cap_rows,
                             const moe_shard_t* shard, const void* w_gate, const void* w_up, const void* w_down,
                             void* h_workspace, void* y_perm, void* workspace, size_t workspace_bytes, uint32_t flags,
                             void* stream) {
  const int st = shard_status(shard);
  if (st != MOE_OK) return st;
  if (cap_rows < 0 || (flags & ~(uint32_t)(MOE_Y_PERM_BF16 | MOE_FFN_SKIP_GATEUP | MOE_FFN_SKIP_DOWN | MOE_FFN_TILED |
                                       MOE_FFN_LEAVE_ROOM)))
    return MOE_ERR_INVALID_ARG;
  if (x == nullptr || expert_offsets == nullptr || w_gate == nullptr || w_up == nullptr ||
      w_down == nullptr || h_workspace == nullptr || y_perm == nullptr)
    return MOE_ERR_INVALID_ARG;
  if (shard->hidden % 64 != 0 || shard->inter_slice % 64 != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (!aligned16(x) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) ||
      !aligned16(h_workspace) || !aligned16(y_perm))
    return MOE_ERR_INVALID_ARG;
  const size_t need = moe_ffn_workspace_bytes(cap_rows, shard);
  if (need > 0 && (workspace == nullptr || workspace_bytes < need || !aligned16(workspace))) return MOE_ERR_WORKSPACE;
  return hip_status(moe::launch_expert_ffn(x, rows, expert_offsets, cap_rows, moe::expected_rows(cap_rows, shard),
                                           shard->n_local_experts, shard->hidden,
                                           shard->inter_slice, w_gate, w_up, w_down, h_workspace, y_perm, workspace,
                                           workspace_bytes, flags, static_cast<hipStream_t>(stream)));
}

int moe_expert_ffn(const void* x_perm, const int32_t* expert_offsets, int32_t cap_rows, const moe_shard_t* shard,
                   const void* w_gate, const void* w_up, const void* w_down, void* h_workspace, void* y_perm,
                   void* workspace, size_t workspace_bytes, uint32_t flags, void* stream) {
  return expert_ffn_common(x_perm, moe::RowMap{nullptr, 1}, expert_offsets, cap_rows, shard, w_gate, w_up, w_down,
                           h_workspace, y_perm, workspace, workspace_bytes, flags, stream);
}

int moe_expert_ffn_gather(const void* x_bf16, const int32_t* row_src, int32_t k, const int32_t* expert_offsets,
                          int32_t cap_rows, const moe_shard_t* shard, const void* w_gate, const void* w_up,
                          const void* w_down, void* h_workspace, void* y_perm, void* workspace,
                          size_t workspace_bytes, uint32_t flags, void* stream) {
  if (row_src == nullptr || k < 1 || k > MOE_MAX_TOPK) return MOE_ERR_INVALID_ARG;
  return expert_ffn_common(x_bf16, moe::RowMap{row_src, k}, expert_offsets, cap_rows, shard, w_gate, w_up, w_down,
                           h_workspace, y_perm, workspace, workspace_bytes, flags, stream);
}

int moe_combine(const void* y_perm, const int32_t* slot_row, const float* topk_w, int32_t T, int32_t k, int32_t H,
                const void* y_shared, const void* x_bf16, const float* w_shared_gate, void* y_out, uint32_t flags,
                void* stream) {
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || H < 8) return MOE_ERR_INVALID_ARG;
  if (flags & ~(uint32_t)(MOE_Y_PERM_BF16 | MOE_OUT_F32)) return MOE_ERR_INVALID_ARG;
  if (y_perm == nullptr || slot_row == nullptr || topk_w == nullptr || y_out == nullptr) return MOE_ERR_INVALID_ARG;
  if ((x_bf16 == nullptr) != (w_shared_gate == nullptr)) return MOE_ERR_INVALID_ARG;
  if (w_shared_gate != nullptr && y_shared == nullptr) return MOE_ERR_INVALID_ARG;
  if (H % 8 != 0) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (!aligned16(y_perm) || !aligned16(y_out) || (y_shared && !aligned16(y_shared)) ||
      (x_bf16 && (!aligned16(x_bf16) || !aligned16(w_shared_gate))))
    return MOE_ERR_INVALID_ARG;
  return hip_status(moe::launch_combine(y_perm, slot_row, topk_w, T, k, H, y_shared, x_bf16, w_shared_gate, y_out,
                                        (flags & MOE_Y_PERM_BF16) != 0, (flags & MOE_OUT_F32) != 0,
                                        static_cast<hipStream_t>(stream)));
}

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_UNSUPPORTED_SHAPE: return "unsupported shape";
    case MOE_ERR_WORKSPACE: return "workspace too small";
    case MOE_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}

}  // extern "C"
