// Grouped "NT" GEMM for decode-sized groups (a few rows per expert): a weight-streaming kernel.
//
// With 1..64 rows per expert the layer is bound by reading every active expert's weights from
// HBM exactly once (paper, "Generative Inference": the decoding stage is memory-bound by weight
// loading), so the design goal is HBM efficiency, not MFMA rate.  This is the generic variant
// (any K that is a multiple of 32, bf16 or fp32 output); grouped_walk.hpp is the faster one for
// the K extents it is instantiated for.
//  * a wavefront streams 16 rows of ONE weight matrix (one MFMA column tile) over its share of K,
//    64 contiguous bytes per row per load, 16-byte loads straight into MFMA operand registers,
//    no LDS on the way.  Measured on MI355X, 16 row streams per wavefront reach ~6.4 TB/s, 32
//    reach ~6.2 and 64 only ~4.5, so the strip is kept at 16 rows;
//  * a workgroup owns (expert, strip of 16 output features).  GEMM1: its 4 wavefronts are
//    {gate, up} x {first, second half of K}; GEMM2: the four quarters of K;
//  * v_mfma_f32_16x16x32_bf16 with the few activation rows as the A operand (rows past the
//    group are clamped to a valid row and never stored): padding M to 16 costs nothing here;
//  * two operand register sets of 4 k-steps in ping-pong keep 4..8 KB of weight loads in flight
//    per wavefront at 4+ wavefronts per SIMD;
//  * the partial accumulators meet in LDS and are summed in a fixed order (deterministic);
//  * experts without rows exit before touching their weights.
#pragma once
#include "moe_internal.hpp"

namespace moe {
namespace gs {

constexpr int kStripN = 16;  // output features per workgroup
constexpr int kWaves = 4;
constexpr int U = 4;         // k32 steps per operand register set
constexpr int kMaxMT = 2;    // 16-row activation tiles handled per pass

__device__ __forceinline__ float silu_mul(float g, float u) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u; }

// Rows [row_lo, row_hi) (at most 16*MT) of one expert against one 16-feature strip.
// red: kWaves * MT * 256 floats of LDS.
template <int MT, bool GATEUP, typename OutT>
__device__ __forceinline__ void stream_rows(float* red, const uint16_t* __restrict__ A, int row_lo, int row_hi,
                                            const uint16_t* __restrict__ Wa, const uint16_t* __restrict__ Wb,
                                            int n0, int n_out, int K, OutT* __restrict__ C, const RowMap rows) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kq = lane >> 4;

  // this wave's matrix and K range, in k32 steps
  const int steps = K / 32;
  const int parts = GATEUP ? 2 : 4;
  const int part = GATEUP ? (wave >> 1) : wave;
  const int s_lo = (steps * part) / parts, s_hi = (steps * (part + 1)) / parts;
  const uint16_t* W = (GATEUP && (wave & 1)) ? Wb : Wa;

  const uint16_t* a_ptr[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) a_ptr[t] = A + (size_t)rows(min(row_lo + t * 16 + l16, row_hi - 1)) * K + kq * 8;
  const uint16_t* b_ptr = W + (size_t)min(n0 + l16, n_out - 1) * K + kq * 8;

  f32x4 acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  struct OperandSet {
    bf16x8 a[U][MT];
    bf16x8 b[U];
  };
  auto load_set = [&](OperandSet& s, int step) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int k = min(step + u, s_hi - 1) * 32;  // steps past the end re-read the last one (unused)
      s.b[u] = *reinterpret_cast<const bf16x8*>(b_ptr + k);
#pragma unroll
      for (int t = 0; t < MT; ++t) s.a[u][t] = *reinterpret_cast<const bf16x8*>(a_ptr[t] + k);
    }
  };
  auto compute_set = [&](const OperandSet& s, int step) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (step + u < s_hi) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(s.a[u][t], s.b[u], acc[t], 0, 0, 0);
      }
    }
  };

  if (s_lo < s_hi) {
    OperandSet s0, s1;
    load_set(s0, s_lo);
    for (int step = s_lo; step < s_hi; step += 2 * U) {
      load_set(s1, step + U);
      compute_set(s0, step);
      load_set(s0, step + 2 * U);
      compute_set(s1, step + U);
    }
  }

  // ---- cross-wave reduction in a fixed order, then the epilogue.  Tile layout in LDS: [row][col].
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    float* dst = red + ((wave * MT + t) << 8);
#pragma unroll
    for (int i = 0; i < 4; ++i) dst[(kq * 4 + i) * 16 + l16] = acc[t][i];
  }
  __syncthreads();
  for (int idx = tid; idx < MT * 256; idx += kWaves * 64) {
    const int t = idx >> 8, r = (idx >> 4) & 15, c = idx & 15;
    const int row = row_lo + t * 16 + r, col = n0 + c;
    const int o = (t << 8) + r * 16 + c;
    const float p0 = red[o], p1 = red[((1 * MT) << 8) + o], p2 = red[((2 * MT) << 8) + o],
                p3 = red[((3 * MT) << 8) + o];
    if (row < row_hi && col < n_out) {
      if constexpr (GATEUP) {  // waves 0,2: gate halves; waves 1,3: up halves
        reinterpret_cast<uint16_t*>(C)[(size_t)row * n_out + col] =
            (uint16_t)f32_to_bf16_bits(silu_mul(p0 + p2, p1 + p3));
      } else if constexpr (sizeof(OutT) == 4) {
        C[(size_t)row * n_out + col] = ((p0 + p1) + p2) + p3;
      } else {
        C[(size_t)row * n_out + col] = (OutT)f32_to_bf16_bits(((p0 + p1) + p2) + p3);
      }
    }
  }
  __syncthreads();
}

constexpr int kRedFloats = kWaves * kMaxMT * 256;  // 16 KB

// grid = (strips, n_local).  GATEUP: Wa = gate, Wb = up [E_loc][n_out][K]; else Wa = down.
// MAXMT = 1 is for launches whose capacity guarantees at most 16 rows per expert: it needs fewer
// registers, so more wavefronts (and more bytes in flight) fit on a CU.
template <int MAXMT, bool GATEUP, typename OutT>
__global__ __launch_bounds__(kWaves * 64) void grouped_stream_kernel(
    const uint16_t* __restrict__ A, const int32_t* __restrict__ expert_offsets, const uint16_t* __restrict__ Wa,
    const uint16_t* __restrict__ Wb, int n_out, int K, OutT* __restrict__ C, const RowMap rows) {
  __shared__ float red[kRedFloats];
  const int e = blockIdx.y;
  const int lo = expert_offsets[e], hi = expert_offsets[e + 1];
  if (hi <= lo) return;  // inactive expert: its weights are never read
  const int n0 = blockIdx.x * kStripN;
  const size_t eoff = (size_t)e * n_out * K;
  const uint16_t* wa = Wa + eoff;
  const uint16_t* wb = GATEUP ? Wb + eoff : nullptr;
  const int M = hi - lo;
  if (MAXMT == 1 || M <= 16) {
    for (int m0 = lo; m0 < hi; m0 += 16)
      stream_rows<1, GATEUP, OutT>(red, A, m0, min(m0 + 16, hi), wa, wb, n0, n_out, K, C, rows);
  } else {
    for (int m0 = lo; m0 < hi; m0 += 32)  // more than 32 rows: the strip is re-streamed per 32 rows
      stream_rows<2, GATEUP, OutT>(red, A, m0, min(m0 + 32, hi), wa, wb, n0, n_out, K, C, rows);
  }
}

}  // namespace gs
}  // namespace moe
