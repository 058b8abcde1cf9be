// Gating network + Top-K selection (paper, "MoE Model Architectures"): router logits in fp32,
// softmax over all experts, k largest logits per token with ties going to the lower expert id.
//
// One wavefront per token.  Logits of expert e live in lane (e % 64), register slot (e / 64),
// so the selection is k wave-wide arg-max reductions and the softmax one wave-wide sum.
#include "moe_internal.hpp"

namespace moe {
namespace {

constexpr int kRouteThreads = 256;
constexpr int kTokPerBlock = kRouteThreads / kWave;
constexpr int kExpChunk = 8;  // experts accumulated per pass over the token's row

template <int EPL>  // expert slots per lane: ceil(E / 64)
__global__ __launch_bounds__(kRouteThreads) void route_topk_kernel(
    const uint16_t* __restrict__ x, const float* __restrict__ w_router, float* __restrict__ logits, int T, int H, int E,
    int k, uint32_t flags, int32_t* __restrict__ topk_idx, float* __restrict__ topk_w) {
  const int lane = threadIdx.x & (kWave - 1);
  const int t = blockIdx.x * kTokPerBlock + (threadIdx.x >> 6);
  if (t >= T) return;

  float myl[EPL];
#pragma unroll
  for (int s = 0; s < EPL; ++s) myl[s] = -INFINITY;

  if (flags & MOE_LOGITS_GIVEN) {
#pragma unroll
    for (int s = 0; s < EPL; ++s) {
      const int e = lane + s * kWave;
      if (e < E) myl[s] = logits[(size_t)t * E + e];
    }
  } else {
    const uint16_t* xr = x + (size_t)t * H;
    for (int e0 = 0; e0 < E; e0 += kExpChunk) {
      float acc[kExpChunk];
#pragma unroll
      for (int j = 0; j < kExpChunk; ++j) acc[j] = 0.f;
      const int ne = min(kExpChunk, E - e0);
      for (int h0 = lane * 8; h0 < H; h0 += kWave * 8) {
        const uint4 xv = *reinterpret_cast<const uint4*>(xr + h0);
        const float xf[8] = {bf16_lo(xv.x), bf16_hi(xv.x), bf16_lo(xv.y), bf16_hi(xv.y),
                             bf16_lo(xv.z), bf16_hi(xv.z), bf16_lo(xv.w), bf16_hi(xv.w)};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float* wr = w_router + (size_t)(h0 + i) * E + e0;
#pragma unroll
          for (int j = 0; j < kExpChunk; ++j)
            if (j < ne) acc[j] = fmaf(xf[i], wr[j], acc[j]);
        }
      }
#pragma unroll
      for (int j = 0; j < kExpChunk; ++j) {
        const float s = wave_sum(acc[j]);
        const int e = e0 + j;
        if (j < ne) {
#pragma unroll
          for (int sl = 0; sl < EPL; ++sl)
            if (sl == (e >> 6) && lane == (e & 63)) myl[sl] = s;
        }
      }
    }
#pragma unroll
    for (int s = 0; s < EPL; ++s) {
      const int e = lane + s * kWave;
      if (e < E) logits[(size_t)t * E + e] = myl[s];
    }
  }

  // k rounds of wave-wide arg-max on (logit desc, expert id asc)
  uint32_t taken = 0;  // bit s set: this lane's slot s already selected
  float sel_v = 0.f;
  int sel_i = 0;
  float vmax = 0.f;
  for (int j = 0; j < k; ++j) {
    float bv = -INFINITY;
    int bi = 0x7FFFFFFF;
#pragma unroll
    for (int s = 0; s < EPL; ++s) {
      const int e = lane + s * kWave;
      if (e < E && !(taken & (1u << s)) && (myl[s] > bv || bi == 0x7FFFFFFF)) {
        bv = myl[s];
        bi = e;
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, kWave);
      const int oi = __shfl_xor(bi, o, kWave);
      const bool take = (oi != 0x7FFFFFFF) && (bi == 0x7FFFFFFF || ov > bv || (ov == bv && oi < bi));
      if (take) {
        bv = ov;
        bi = oi;
      }
    }
    if ((bi & 63) == lane) taken |= 1u << (bi >> 6);
    if (j == 0) vmax = bv;
    if (lane == j) {
      sel_v = bv;
      sel_i = bi;
    }
  }

  // softmax denominator over all E experts (max logit is the first selected one)
  float part = 0.f;
#pragma unroll
  for (int s = 0; s < EPL; ++s) {
    const int e = lane + s * kWave;
    if (e < E) part += expf(myl[s] - vmax);
  }
  const float denom_all = wave_sum(part);
  const float num = (lane < k) ? expf(sel_v - vmax) : 0.f;
  const float denom_sel = wave_sum(num);
  if (lane < k) {
    const float w = num / ((flags & MOE_RENORM_TOPK) ? denom_sel : denom_all);
    topk_idx[(size_t)t * k + lane] = sel_i;
    topk_w[(size_t)t * k + lane] = w;
  }
}

}  // namespace

hipError_t launch_route_topk(const void* x, const float* w_router, float* logits, int T, int H, int E, int k,
                             uint32_t flags, int32_t* topk_idx, float* topk_w, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  const dim3 grid((T + kTokPerBlock - 1) / kTokPerBlock), block(kRouteThreads);
  const uint16_t* xs = static_cast<const uint16_t*>(x);
  const int epl = (E + kWave - 1) / kWave;
  switch (epl) {
    case 1:
      hipLaunchKernelGGL(route_topk_kernel<1>, grid, block, 0, stream, xs, w_router, logits, T, H, E, k, flags,
                         topk_idx, topk_w);
      break;
    case 2:
      hipLaunchKernelGGL(route_topk_kernel<2>, grid, block, 0, stream, xs, w_router, logits, T, H, E, k, flags,
                         topk_idx, topk_w);
      break;
    default:
      hipLaunchKernelGGL(route_topk_kernel<4>, grid, block, 0, stream, xs, w_router, logits, T, H, E, k, flags,
                         topk_idx, topk_w);
      break;
  }
  return hipGetLastError();
}

}  // namespace moe
