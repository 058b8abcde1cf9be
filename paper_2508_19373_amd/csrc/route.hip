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

// Top-K selection and gate weights of one token by one wavefront.  myl[s] holds the logit of
// expert lane + 64*s (-inf past E).  k rounds of wave-wide arg-max on (logit desc, expert id asc),
// then softmax over all E logits evaluated at the selected ones.
template <int EPL>
__device__ __forceinline__ void select_topk(const float (&myl)[EPL], int lane, int E, int k, uint32_t flags,
                                            int32_t* __restrict__ idx_out, float* __restrict__ w_out) {
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
    idx_out[lane] = sel_i;
    w_out[lane] = num / ((flags & MOE_RENORM_TOPK) ? denom_sel : denom_all);
  }
}

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

  select_topk<EPL>(myl, lane, E, k, flags, topk_idx + (size_t)t * k, topk_w + (size_t)t * k);
}

// Router logits as a small fp32 MFMA GEMM: logits[16 tokens, 16 experts] tiles with
// v_mfma_f32_16x16x4_f32 (x is widened bf16 -> fp32 exactly, W_r is read as it is laid out,
// [H,E] row-major = the B operand's natural k-major form).  A workgroup owns 16 tokens; its NWV
// wavefronts split the hidden dimension in 32-wide chunks (UNR chunks' loads are issued before
// their MFMAs, so a decode-sized call is a couple of memory round trips, not one per chunk) and
// the partial tiles are summed in wave order through LDS; the same workgroup then selects the
// top k of its 16 tokens from the logits tile, one wavefront per token.  The sum over k may be taken in any
// order, so one 16-byte load per lane feeds 8 MFMAs: in MFMA s, lane (m, kq) supplies
// x[t0+m, c*32 + kq*8 + s] and the B lane (n, kq) the matching W_r row.
constexpr int kLogitTok = 16;

// SELECT = false (decode-sized batches with more than 16 experts): grid.y walks the 16-expert
// column tiles, one per workgroup, so that a batch of 32 tokens is spread over 2 x E/16 workgroups
// instead of 2; the logits go to global memory and route_topk_kernel selects from there.
template <int NT, int NWV, int UNR, bool SELECT>  // 16-expert column tiles, wavefronts, chunks in flight per wavefront
__global__ __launch_bounds__(NWV * 64) void router_logits_kernel(const uint16_t* __restrict__ x,
                                                                 const float* __restrict__ w_router,
                                                                 float* __restrict__ logits, int T, int H, int E,
                                                                 int k, uint32_t flags,
                                                                 int32_t* __restrict__ topk_idx,
                                                                 float* __restrict__ topk_w) {
  __shared__ float part[NWV][NT][16][17];
  __shared__ float tile[16][NT * 16 + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t0 = blockIdx.x * kLogitTok;
  const int e_base = SELECT ? 0 : blockIdx.y * (NT * 16);
  const int m = lane & 15, kq = lane >> 4;
  const int trow = min(t0 + m, T - 1);
  const uint16_t* xr = x + (size_t)trow * H + kq * 8;
  f32x4 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int n_chunks = H / 32;
  for (int c0 = wave; c0 < n_chunks; c0 += NWV * UNR) {
    uint4 xv[UNR];
    float wv[UNR][8][NT];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int c = min(c0 + u * NWV, n_chunks - 1);  // past the end: re-read, weight forced to 0 below
      const bool live = c0 + u * NWV < n_chunks;
      xv[u] = *reinterpret_cast<const uint4*>(xr + c * 32);
      const float* wr = w_router + (size_t)(c * 32 + kq * 8) * E + e_base + m;
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wv[u][s][nt] = (live && e_base + nt * 16 + m < E) ? wr[(size_t)s * E + nt * 16] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const float xf[8] = {bf16_lo(xv[u].x), bf16_hi(xv[u].x), bf16_lo(xv[u].y), bf16_hi(xv[u].y),
                           bf16_lo(xv[u].z), bf16_hi(xv[u].z), bf16_lo(xv[u].w), bf16_hi(xv[u].w)};
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(xf[s], wv[u][s][nt], acc[nt], 0, 0, 0);
    }
  }
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int i = 0; i < 4; ++i) part[wave][nt][kq * 4 + i][m] = acc[nt][i];
  __syncthreads();
  for (int idx = tid; idx < NT * 256; idx += NWV * 64) {
    const int nt = idx >> 8, row = (idx >> 4) & 15, col = idx & 15;
    const int e = e_base + nt * 16 + col, t = t0 + row;
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; ++w) sum += part[w][nt][row][col];
    tile[row][nt * 16 + col] = sum;
    if (e < E && t < T) logits[(size_t)t * E + e] = sum;
  }
  if constexpr (!SELECT) return;
  __syncthreads();
  // selection: one wavefront per token, straight from the logits tile in LDS
  constexpr int EPL = (NT * 16 + kWave - 1) / kWave;
  for (int row = wave; row < 16; row += NWV) {
    const int t = t0 + row;
    if (t >= T) break;
    float myl[EPL];
#pragma unroll
    for (int s = 0; s < EPL; ++s) {
      const int e = lane + s * kWave;
      myl[s] = (e < E) ? tile[row][e] : -INFINITY;
    }
    select_topk<EPL>(myl, lane, E, k, flags, topk_idx + (size_t)t * k, topk_w + (size_t)t * k);
  }
}

// Decode-sized batches with 8 experts: one workgroup per token on the vector units.  The MFMA
// kernel above puts 16 tokens on one compute unit, 3.4 us of fp32 matrix work at H = 4096 behind
// two memory round trips, whatever the batch; here a token's row is spread over 256 lanes (8 hidden
// values each per step, their W_r rows fetched as 16-byte vectors), the E partial sums are added
// across the lanes and wavefronts in a fixed order, and wavefront 0 selects.  E4 = E / 4.
template <int E4>
__global__ __launch_bounds__(256) void route_small_kernel(const uint16_t* __restrict__ x,
                                                          const float* __restrict__ w_router,
                                                          float* __restrict__ logits, int H, int k, uint32_t flags,
                                                          int32_t* __restrict__ topk_idx,
                                                          float* __restrict__ topk_w) {
  constexpr int E = E4 * 4;
  __shared__ float part[4][E];
  const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;
  const uint16_t* xr = x + (size_t)t * H;
  for (int h0 = tid * 8; h0 < H; h0 += 256 * 8) {
    const uint4 xv = *reinterpret_cast<const uint4*>(xr + h0);
    const float xf[8] = {bf16_lo(xv.x), bf16_hi(xv.x), bf16_lo(xv.y), bf16_hi(xv.y),
                         bf16_lo(xv.z), bf16_hi(xv.z), bf16_lo(xv.w), bf16_hi(xv.w)};
    const float4* wr = reinterpret_cast<const float4*>(w_router + (size_t)h0 * E);
    float4 wv[8][E4];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int q = 0; q < E4; ++q) wv[i][q] = wr[i * E4 + q];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int q = 0; q < E4; ++q) {
        acc[q * 4 + 0] = fmaf(xf[i], wv[i][q].x, acc[q * 4 + 0]);
        acc[q * 4 + 1] = fmaf(xf[i], wv[i][q].y, acc[q * 4 + 1]);
        acc[q * 4 + 2] = fmaf(xf[i], wv[i][q].z, acc[q * 4 + 2]);
        acc[q * 4 + 3] = fmaf(xf[i], wv[i][q].w, acc[q * 4 + 3]);
      }
  }
#pragma unroll
  for (int e = 0; e < E; ++e) {
    const float s = wave_sum(acc[e]);
    if (lane == 0) part[wave][e] = s;
  }
  __syncthreads();
  if (wave != 0) return;
  float myl[1];
  myl[0] = lane < E ? ((part[0][min(lane, E - 1)] + part[1][min(lane, E - 1)]) + part[2][min(lane, E - 1)]) +
                          part[3][min(lane, E - 1)]
                    : -INFINITY;
  if (lane < E) logits[(size_t)t * E + lane] = myl[0];
  select_topk<1>(myl, lane, E, k, flags, topk_idx + (size_t)t * k, topk_w + (size_t)t * k);
}

template <int NT, int NWV, int UNR>
void launch_logits(const uint16_t* x, const float* w_router, float* logits, int T, int H, int E, int k, uint32_t flags,
                   int32_t* topk_idx, float* topk_w, hipStream_t stream) {
  hipLaunchKernelGGL((router_logits_kernel<NT, NWV, UNR, true>), dim3((T + kLogitTok - 1) / kLogitTok),
                     dim3(NWV * 64), 0, stream, x, w_router, logits, T, H, E, k, flags, topk_idx, topk_w);
}

}  // namespace

hipError_t launch_route_topk(const void* x, const float* w_router, float* logits, int T, int H, int E, int k,
                             uint32_t flags, int32_t* topk_idx, float* topk_w, hipStream_t stream) {
  if (T == 0) return hipSuccess;
  const dim3 grid((T + kTokPerBlock - 1) / kTokPerBlock), block(kRouteThreads);
  const uint16_t* xs = static_cast<const uint16_t*>(x);
  if (!(flags & MOE_LOGITS_GIVEN) && H % 32 == 0) {
    const int nt = (E + 15) / 16;
    // (measured at H = 4096, 1 to 64 tokens: 8.5 against 11.5 us with 8 experts; with 16 experts the
    // MFMA kernel stays ahead, 11.7 against 12.9 us)
    if (T <= 64 && E == 8 && (reinterpret_cast<uintptr_t>(w_router) & 15u) == 0) {
      hipLaunchKernelGGL(route_small_kernel<2>, dim3(T), dim3(256), 0, stream, xs, w_router, logits, H, k, flags,
                         topk_idx, topk_w);
      return hipGetLastError();
    }
    if (nt < 2 || T > 1024) {  // logits by MFMA and the selection from the logits tile, in one kernel
      if (nt <= 1) launch_logits<1, 16, 4>(xs, w_router, logits, T, H, E, k, flags, topk_idx, topk_w, stream);
      else if (nt <= 2) launch_logits<2, 16, 4>(xs, w_router, logits, T, H, E, k, flags, topk_idx, topk_w, stream);
      else if (nt <= 4) launch_logits<4, 16, 2>(xs, w_router, logits, T, H, E, k, flags, topk_idx, topk_w, stream);
      else if (nt <= 8) launch_logits<8, 8, 1>(xs, w_router, logits, T, H, E, k, flags, topk_idx, topk_w, stream);
      else launch_logits<16, 4, 1>(xs, w_router, logits, T, H, E, k, flags, topk_idx, topk_w, stream);
      return hipGetLastError();
    }
    // up to 1024 tokens and more than 16 experts: one workgroup per (16 tokens, 16 experts), then select
    // from the logits (measured at 60 experts: 11 against 21 us at 256 and 1024 tokens, 31 against 24 us at 4096)
    hipLaunchKernelGGL((router_logits_kernel<1, 16, 4, false>), dim3((T + kLogitTok - 1) / kLogitTok, nt),
                       dim3(16 * 64), 0, stream, xs, w_router, logits, T, H, E, k, flags, topk_idx, topk_w);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
    flags |= MOE_LOGITS_GIVEN;
  }
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
