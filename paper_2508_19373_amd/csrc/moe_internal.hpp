// Internal declarations shared by the HIP translation units of libmoe_shard (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_shard.h"

namespace moe {

constexpr int kWave = 64;

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// bf16 bit pattern <-> fp32
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xFFFF0000u); }

// fp32 -> bf16, round to nearest even, by the hardware converter (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return *reinterpret_cast<const uint32_t*>(&b);
}
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) { return pack_bf16x2(f, 0.f) & 0xFFFFu; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// Where the rows of the first GEMM come from: row r of the input is x[row_src[r] / k] (the token of
// assignment row_src[r]); row_src == nullptr means the input is already permuted (row r itself).
struct RowMap {
  const int32_t* row_src;
  int k;
  __host__ __device__ inline int operator()(int r) const { return row_src ? row_src[r] / k : r; }
};

// launchers (each returns hipGetLastError() after enqueueing on `stream`)
hipError_t launch_route_topk(const void* x, const float* w_router, float* logits, int T, int H, int E, int k,
                             uint32_t flags, int32_t* topk_idx, float* topk_w, hipStream_t stream);
hipError_t launch_permute(const void* x, const int32_t* topk_idx, int T, int k, int H, int n_local, int offset,
                          void* x_perm, int32_t* expert_offsets, int32_t* row_src, int32_t* slot_row,
                          void* workspace, hipStream_t stream);
size_t permute_workspace_bytes(int T, int k, int n_local);
// The same with the library's own static scratch; permute_static_counts: int32 counts it would use.
hipError_t launch_permute_static(const void* x, const int32_t* topk_idx, int T, int k, int H, int n_local, int offset,
                                 void* x_perm, int32_t* expert_offsets, int32_t* row_src, int32_t* slot_row,
                                 hipStream_t stream);
size_t permute_static_counts(int T, int k, int n_local);
// est_rows: the rows this shard expects (cap_rows scaled by its share of the experts); it steers the
// choice of kernels and K slices only, every bound is taken from cap_rows.
hipError_t launch_expert_ffn(const void* x_perm, RowMap rows, const int32_t* expert_offsets, int cap_rows, int est_rows,
                             int n_local, int H, int I_s, const void* w_gate, const void* w_up, const void* w_down,
                             void* h_ws, void* y_perm, void* workspace, size_t workspace_bytes, uint32_t flags,
                             hipStream_t stream);
size_t ffn_workspace_bytes(int cap_rows, int est_rows, int n_local, int H, int I_s);
// What launch_expert_ffn would do: {GEMM1 by the walk kernel, GEMM2 by the walk kernel, rows per
// walk pass / 16, K slices of GEMM2}.
void ffn_plan(int cap_rows, int est_rows, int n_local, int H, int I_s, int32_t out[4]);
// Row-block height of the tiled kernels for such a call (256, or 160 for the one-height work list).
int tiled_block_rows(int cap_rows, int est_rows, int n_local, int H, int I_s);
int expected_rows(int cap_rows, const moe_shard_t* shard);
hipError_t launch_combine(const void* y_perm, const int32_t* slot_row, const float* topk_w, int T, int k, int H,
                          const void* y_shared, const void* x, const float* w_shared_gate, void* y_out,
                          bool y_perm_bf16, bool out_f32, hipStream_t stream);

}  // namespace moe
