// INT4 per-group backup of expert weights: dequantise to bf16 (the step on the paper's strategy
// switching path, "The Dynamic Parallelism Transition Strategy") and quantise (builds the backup).
//
// Both kernels are pure streaming: dequantise reads 0.5625 bytes and writes 2 bytes per weight, so
// the design goal is HBM efficiency.  A lane handles 8 consecutive weights: one 4-byte load of
// codes, one 16-byte store of bf16 (both fully coalesced across the wavefront); the 8 lanes of a
// group share one 4-byte (scale, min) word, which the first of them pulls into the L1.  Four
// independent items per lane keep enough loads in flight.
#include "moe_int4.h"
#include "moe_internal.hpp"

namespace moe {
namespace {

constexpr int kThreads = 256;
constexpr int kItems = 4;                                  // 8-weight items per lane
constexpr int64_t kBlockWeights = (int64_t)kThreads * kItems * 8;  // 8192

__global__ __launch_bounds__(kThreads) void int4_dequantize_kernel(const uint32_t* __restrict__ codes,
                                                                   const uint32_t* __restrict__ qparams,
                                                                   int64_t n_items, uint4* __restrict__ out) {
  const int64_t base = (int64_t)blockIdx.x * (kThreads * kItems) + threadIdx.x;
  uint32_t c[kItems], qp[kItems];
#pragma unroll
  for (int it = 0; it < kItems; ++it) {
    const int64_t i = base + it * kThreads;
    if (i < n_items) {
      c[it] = __builtin_nontemporal_load(codes + i);
      qp[it] = qparams[i >> 3];
    }
  }
#pragma unroll
  for (int it = 0; it < kItems; ++it) {
    const int64_t i = base + it * kThreads;
    if (i < n_items) {
      const float scale = bf16_lo(qp[it]), mn = bf16_hi(qp[it]);
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = fmaf((float)((c[it] >> (4 * j)) & 15u), scale, mn);
      uint4 o;
      o.x = pack_bf16x2(v[0], v[1]);
      o.y = pack_bf16x2(v[2], v[3]);
      o.z = pack_bf16x2(v[4], v[5]);
      o.w = pack_bf16x2(v[6], v[7]);
      __builtin_nontemporal_store(o.x, &out[i].x);
      __builtin_nontemporal_store(o.y, &out[i].y);
      __builtin_nontemporal_store(o.z, &out[i].z);
      __builtin_nontemporal_store(o.w, &out[i].w);
    }
  }
}

// 8 lanes per group: each loads 8 weights (16 bytes), min / max meet by three butterfly steps.
__global__ __launch_bounds__(kThreads) void int4_quantize_kernel(const uint4* __restrict__ w, int64_t n_items,
                                                                 uint32_t* __restrict__ codes,
                                                                 uint32_t* __restrict__ qparams) {
  const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  // n_items is a multiple of 8, so the 8 lanes of a group are in range together
  const bool live = i < n_items;
  uint4 raw = make_uint4(0, 0, 0, 0);
  if (live) raw = w[i];
  float v[8] = {bf16_lo(raw.x), bf16_hi(raw.x), bf16_lo(raw.y), bf16_hi(raw.y),
                bf16_lo(raw.z), bf16_hi(raw.z), bf16_lo(raw.w), bf16_hi(raw.w)};
  float mn = v[0], mx = v[0];
#pragma unroll
  for (int j = 1; j < 8; ++j) {
    mn = fminf(mn, v[j]);
    mx = fmaxf(mx, v[j]);
  }
#pragma unroll
  for (int o = 1; o < 8; o <<= 1) {
    mn = fminf(mn, __shfl_xor(mn, o, kWave));
    mx = fmaxf(mx, __shfl_xor(mx, o, kWave));
  }
  const uint32_t scale_bits = f32_to_bf16_bits((mx - mn) / 15.0f);
  const float scale = bf16_bits_to_f32(scale_bits);
  uint32_t packed = 0;
  if (scale > 0.f) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float q = rintf((v[j] - mn) / scale);
      q = fminf(fmaxf(q, 0.f), 15.f);
      packed |= (uint32_t)q << (4 * j);
    }
  }
  if (live) {
    codes[i] = packed;
    if ((i & 7) == 0) qparams[i >> 3] = scale_bits | (__float_as_uint(mn) & 0xFFFF0000u);  // mn is a bf16 value
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace
}  // namespace moe

extern "C" {

int moe_int4_dequantize(const void* codes, const void* qparams, int64_t n_elems, void* w_bf16, void* stream) {
  using namespace moe;
  if (n_elems < 0 || n_elems % MOE_INT4_GROUP != 0) return MOE_ERR_INVALID_ARG;
  if (codes == nullptr || qparams == nullptr || w_bf16 == nullptr) return MOE_ERR_INVALID_ARG;
  if (!aligned16(codes) || !aligned16(qparams) || !aligned16(w_bf16)) return MOE_ERR_INVALID_ARG;
  if (n_elems / kBlockWeights >= 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (n_elems == 0) return MOE_OK;
  const int64_t n_items = n_elems / 8;
  const unsigned grid = (unsigned)((n_elems + kBlockWeights - 1) / kBlockWeights);
  hipLaunchKernelGGL(int4_dequantize_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint32_t*>(codes), static_cast<const uint32_t*>(qparams), n_items,
                     static_cast<uint4*>(w_bf16));
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

int moe_int4_quantize(const void* w_bf16, int64_t n_elems, void* codes, void* qparams, void* stream) {
  using namespace moe;
  if (n_elems < 0 || n_elems % MOE_INT4_GROUP != 0) return MOE_ERR_INVALID_ARG;
  if (codes == nullptr || qparams == nullptr || w_bf16 == nullptr) return MOE_ERR_INVALID_ARG;
  if (!aligned16(codes) || !aligned16(qparams) || !aligned16(w_bf16)) return MOE_ERR_INVALID_ARG;
  const int64_t n_items = n_elems / 8;
  if ((n_items + kThreads - 1) / kThreads >= 0x7FFFFFFF) return MOE_ERR_UNSUPPORTED_SHAPE;
  if (n_elems == 0) return MOE_OK;
  const unsigned grid = (unsigned)((n_items + kThreads - 1) / kThreads);
  hipLaunchKernelGGL(int4_quantize_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(w_bf16), n_items, static_cast<uint32_t*>(codes),
                     static_cast<uint32_t*>(qparams));
  return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP;
}

}  // extern "C"
