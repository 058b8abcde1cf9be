// Weighted un-permute / combine of the Top-K expert outputs (paper, "MoE Model Architectures":
// each token's result is the gate-weighted mix of its selected experts), plus the always-active
// shared expert scaled by sigmoid(x . w_s).
//
// Token-major gather: one workgroup per token walks the token's k slots in order and sums in
// fp32, so every output row is written exactly once, coalesced, with no atomics -- the result
// is deterministic.  HBM-bound: reads k rows of y_perm, writes one row of y.
#include "moe_internal.hpp"

namespace moe {
namespace {

constexpr int kCombThreads = 256;

__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const uint16_t* p, float (&v)[8]) {
  const uint4 a = *reinterpret_cast<const uint4*>(p);
  v[0] = bf16_lo(a.x); v[1] = bf16_hi(a.x); v[2] = bf16_lo(a.y); v[3] = bf16_hi(a.y);
  v[4] = bf16_lo(a.z); v[5] = bf16_hi(a.z); v[6] = bf16_lo(a.w); v[7] = bf16_hi(a.w);
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(uint16_t* p, const float (&v)[8]) {
  uint4 o;
  o.x = pack_bf16x2(v[0], v[1]);
  o.y = pack_bf16x2(v[2], v[3]);
  o.z = pack_bf16x2(v[4], v[5]);
  o.w = pack_bf16x2(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = o;
}

template <typename YT, typename OT>
__global__ __launch_bounds__(kCombThreads) void combine_kernel(const YT* __restrict__ y_perm,
                                                              const int32_t* __restrict__ slot_row,
                                                              const float* __restrict__ topk_w, int T, int k, int H,
                                                              const YT* __restrict__ y_shared,
                                                              const uint16_t* __restrict__ x,
                                                              const float* __restrict__ w_shared_gate,
                                                              OT* __restrict__ y_out) {
  __shared__ float red[kCombThreads / kWave];
  __shared__ int s_row[MOE_MAX_TOPK];
  __shared__ float s_w[MOE_MAX_TOPK];
  const int tid = threadIdx.x;
  for (int t = blockIdx.x; t < T; t += gridDim.x) {
    __syncthreads();  // LDS reuse across tokens
    if (tid < k) {
      s_row[tid] = slot_row[(size_t)t * k + tid];
      s_w[tid] = topk_w[(size_t)t * k + tid];
    }
    float gate = 1.f;
    if (y_shared != nullptr && w_shared_gate != nullptr) {
      float part = 0.f;
      for (int h0 = tid * 8; h0 < H; h0 += kCombThreads * 8) {
        float xv[8], wv[8];
        load8(x + (size_t)t * H + h0, xv);
        load8(w_shared_gate + h0, wv);
#pragma unroll
        for (int i = 0; i < 8; ++i) part = fmaf(xv[i], wv[i], part);
      }
      part = wave_sum(part);
      if ((tid & (kWave - 1)) == 0) red[tid >> 6] = part;
      __syncthreads();
      float z = 0.f;
#pragma unroll
      for (int w = 0; w < kCombThreads / kWave; ++w) z += red[w];
      gate = 1.f / (1.f + expf(-z));
    } else {
      __syncthreads();
    }
    for (int h0 = tid * 8; h0 < H; h0 += kCombThreads * 8) {
      float acc[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = 0.f;
      for (int j = 0; j < k; ++j) {
        const int r = s_row[j];
        if (r < 0) continue;
        const float w = s_w[j];
        float v[8];
        load8(y_perm + (size_t)r * H + h0, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(w, v[i], acc[i]);
      }
      if (y_shared != nullptr) {
        float v[8];
        load8(y_shared + (size_t)t * H + h0, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(gate, v[i], acc[i]);
      }
      store8(y_out + (size_t)t * H + h0, acc);
    }
  }
}

template <typename YT, typename OT>
hipError_t launch_typed(const void* y_perm, const int32_t* slot_row, const float* topk_w, int T, int k, int H,
                        const void* y_shared, const void* x, const float* w_shared_gate, void* y_out,
                        hipStream_t stream) {
  const int grid = T < 16384 ? T : 16384;
  hipLaunchKernelGGL((combine_kernel<YT, OT>), dim3(grid), dim3(kCombThreads), 0, stream,
                     static_cast<const YT*>(y_perm), slot_row, topk_w, T, k, H, static_cast<const YT*>(y_shared),
                     static_cast<const uint16_t*>(x), w_shared_gate, static_cast<OT*>(y_out));
  return hipGetLastError();
}

}  // namespace

hipError_t launch_combine(const void* y_perm, const int32_t* slot_row, const float* topk_w, int T, int k, int H,
                          const void* y_shared, const void* x, const float* w_shared_gate, void* y_out,
                          bool y_perm_bf16, bool out_f32, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  if (y_perm_bf16) {
    return out_f32 ? launch_typed<uint16_t, float>(y_perm, slot_row, topk_w, T, k, H, y_shared, x, w_shared_gate,
                                                   y_out, stream)
                   : launch_typed<uint16_t, uint16_t>(y_perm, slot_row, topk_w, T, k, H, y_shared, x, w_shared_gate,
                                                      y_out, stream);
  }
  return out_f32
             ? launch_typed<float, float>(y_perm, slot_row, topk_w, T, k, H, y_shared, x, w_shared_gate, y_out, stream)
             : launch_typed<float, uint16_t>(y_perm, slot_row, topk_w, T, k, H, y_shared, x, w_shared_gate, y_out,
                                             stream);
}

}  // namespace moe
