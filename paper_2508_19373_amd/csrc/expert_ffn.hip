// Expert networks on the permuted rows (paper, "MoE Model Architectures": the Expert module's
// parallel expert networks, evaluated only for the tokens the gating network sent to them;
// "Tensor Parallelism": a shard may hold only a slice of the intermediate dimension, in which
// case the result is the unreduced partial sum).
//
// Two grouped GEMMs, both "NT" (activations and weights are K-contiguous):
//   GEMM1  h[r, i]  = silu(x_r . Wg_e[i,:]) * (x_r . Wu_e[i,:])      K = H,   N = I_s (gate+up fused)
//   GEMM2  y[r, n]  = h_r . Wd_e[n,:]                                K = I_s, N = H
// bf16 operands, v_mfma_f32_32x32x16_bf16, fp32 accumulators.  A workgroup owns one
// (expert, row block, column block) tile; row blocks never straddle two experts, so the tile
// list is derived on the device from expert_offsets without a host round trip.
#include "grouped_gemm.hpp"
#include "moe_internal.hpp"

namespace moe {
namespace {

constexpr int BK = 64;  // K elements per LDS tile row: 128 bytes = 8 chunks of 16 bytes

// LDS tiles are [rows][64] bf16.  The 16-byte chunk index of a row is XOR-ed with (row/2)%8 so
// that the 32 rows an MFMA operand read touches at one k offset spread over all banks.
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * BK + ((chunk ^ ((row >> 1) & 7)) << 3); }

// Row of accumulator register i in lane `lane` of a 32x32 MFMA result tile (column = lane % 32).
__device__ __forceinline__ int acc_row(int i, int lane) { return ((i >> 2) << 3) + ((lane >> 5) << 2) + (i & 3); }

__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.f + __expf(-g)) * u; }

template <int BM, int BN, int WM, int WN, bool GATEUP, typename OutT>
__global__ __launch_bounds__(WM* WN * 64) void grouped_gemm_kernel(
    const uint16_t* __restrict__ A, const int32_t* __restrict__ expert_offsets, int n_local, int cap_rows,
    const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1, int n_out, int K, OutT* __restrict__ C) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int A_LD = BM * 8 / NT, B_LD = BN * 8 / NT;
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile / wave grid mismatch");
  static_assert((BM * 8) % NT == 0 && (BN * 8) % NT == 0, "loader mismatch");
  static_assert(!GATEUP || (TN % 2 == 0), "gate and up column blocks must pair up inside a wave");
  constexpr int NCOLS = GATEUP ? BN / 2 : BN;  // output columns per tile

  __shared__ __attribute__((aligned(16))) uint16_t sA[2][BM * BK];
  __shared__ __attribute__((aligned(16))) uint16_t sB[2][BN * BK];

  // ---- which (expert, row block) is this?
  int mb = blockIdx.y, e = 0, lo = 0, hi = 0;
  bool found = false;
  for (e = 0; e < n_local; ++e) {
    lo = expert_offsets[e];
    hi = expert_offsets[e + 1];
    const int nb = (hi - lo + BM - 1) / BM;
    if (mb < nb) {
      found = true;
      break;
    }
    mb -= nb;
  }
  if (!found) return;
  const int row0 = lo + mb * BM;
  const int col0 = blockIdx.x * NCOLS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- global -> register -> LDS loaders: thread handles chunk (tid % 8) of rows tid/8 + i*NT/8
  const uint16_t* a_ptr[A_LD];
  const uint16_t* b_ptr[B_LD];
  int a_lds[A_LD], b_lds[B_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) {
    const int r = (tid >> 3) + i * (NT / 8), c = tid & 7;
    const int gr = min(row0 + r, cap_rows - 1);  // rows past the group are read but never stored
    a_ptr[i] = A + (size_t)gr * K + c * 8;
    a_lds[i] = lds_off(r, c);
  }
  const size_t expert_stride = (size_t)n_out * K;
#pragma unroll
  for (int i = 0; i < B_LD; ++i) {
    const int r = (tid >> 3) + i * (NT / 8), c = tid & 7;
    const uint16_t* base;
    int wrow;
    if (GATEUP) {  // 32-row blocks alternate gate, up, gate, up ... of the same output columns
      const int jb = r >> 5;
      wrow = col0 + (jb >> 1) * 32 + (r & 31);
      base = (jb & 1) ? B1 : B0;
    } else {
      wrow = col0 + r;
      base = B0;
    }
    wrow = min(wrow, n_out - 1);
    b_ptr[i] = base + (size_t)e * expert_stride + (size_t)wrow * K + c * 8;
    b_lds[i] = lds_off(r, c);
  }

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint4 a_reg[A_LD], b_reg[B_LD];
#pragma unroll
  for (int i = 0; i < A_LD; ++i) a_reg[i] = *reinterpret_cast<const uint4*>(a_ptr[i]);
#pragma unroll
  for (int i = 0; i < B_LD; ++i) b_reg[i] = *reinterpret_cast<const uint4*>(b_ptr[i]);
#pragma unroll
  for (int i = 0; i < A_LD; ++i) *reinterpret_cast<uint4*>(&sA[0][a_lds[i]]) = a_reg[i];
#pragma unroll
  for (int i = 0; i < B_LD; ++i) *reinterpret_cast<uint4*>(&sB[0][b_lds[i]]) = b_reg[i];
  __syncthreads();

  const int nk = K / BK;
  const int a_row = wm * (BM / WM) + (lane & 31);
  const int b_row = wn * (BN / WN) + (lane & 31);
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < A_LD; ++i) a_reg[i] = *reinterpret_cast<const uint4*>(a_ptr[i] + (size_t)(kt + 1) * BK);
#pragma unroll
      for (int i = 0; i < B_LD; ++i) b_reg[i] = *reinterpret_cast<const uint4*>(b_ptr[i] + (size_t)(kt + 1) * BK);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int c = ks * 2 + (lane >> 5);
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = *reinterpret_cast<const bf16x8*>(&sA[cur][lds_off(a_row + i * 32, c)]);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = *reinterpret_cast<const bf16x8*>(&sB[cur][lds_off(b_row + j * 32, c)]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
#pragma unroll
      for (int i = 0; i < A_LD; ++i) *reinterpret_cast<uint4*>(&sA[cur ^ 1][a_lds[i]]) = a_reg[i];
#pragma unroll
      for (int i = 0; i < B_LD; ++i) *reinterpret_cast<uint4*>(&sB[cur ^ 1][b_lds[i]]) = b_reg[i];
    }
    __syncthreads();
  }

  // ---- epilogue
  const int lcol = lane & 31;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int rbase = row0 + wm * (BM / WM) + i * 32;
    if (GATEUP) {
#pragma unroll
      for (int j = 0; j < TN; j += 2) {
        const int jb = wn * TN + j;  // even: gate block; jb + 1: up block of the same columns
        const int col = col0 + (jb >> 1) * 32 + lcol;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rbase + acc_row(v, lane);
          if (row < hi && col < n_out) {
            const float hval = silu_mul(acc[i][j][v], acc[i][j + 1][v]);
            reinterpret_cast<uint16_t*>(C)[(size_t)row * n_out + col] = (uint16_t)f32_to_bf16_bits(hval);
          }
        }
      }
    } else {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col0 + wn * (BN / WN) + j * 32 + lcol;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = rbase + acc_row(v, lane);
          if (row < hi && col < n_out) {
            if constexpr (sizeof(OutT) == 4)
              C[(size_t)row * n_out + col] = acc[i][j][v];
            else
              C[(size_t)row * n_out + col] = (OutT)f32_to_bf16_bits(acc[i][j][v]);
          }
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_pair(const void* x_perm, const int32_t* expert_offsets, int cap_rows, int n_local, int H, int I_s,
                       const void* w_gate, const void* w_up, const void* w_down, void* h_ws, void* y_perm,
                       uint32_t flags, hipStream_t stream) {
  const bool y_bf16 = (flags & MOE_Y_PERM_BF16) != 0;
  const int m_blocks = cap_rows / BM + n_local;  // upper bound on sum_e ceil(rows_e / BM)
  const dim3 block(WM * WN * 64);
  const uint16_t* xp = static_cast<const uint16_t*>(x_perm);
  uint16_t* hw = static_cast<uint16_t*>(h_ws);
  if (!(flags & MOE_FFN_SKIP_GATEUP)) {
    const dim3 grid((I_s + BN / 2 - 1) / (BN / 2), m_blocks);
    hipLaunchKernelGGL((grouped_gemm_kernel<BM, BN, WM, WN, true, uint16_t>), grid, block, 0, stream, xp,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_gate),
                       static_cast<const uint16_t*>(w_up), I_s, H, hw);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  if (flags & MOE_FFN_SKIP_DOWN) return hipSuccess;
  const dim3 grid((H + BN - 1) / BN, m_blocks);
  if (y_bf16)
    hipLaunchKernelGGL((grouped_gemm_kernel<BM, BN, WM, WN, false, uint16_t>), grid, block, 0, stream, hw,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_down),
                       static_cast<const uint16_t*>(nullptr), H, I_s, static_cast<uint16_t*>(y_perm));
  else
    hipLaunchKernelGGL((grouped_gemm_kernel<BM, BN, WM, WN, false, float>), grid, block, 0, stream, hw,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_down),
                       static_cast<const uint16_t*>(nullptr), H, I_s, static_cast<float*>(y_perm));
  return hipGetLastError();
}

// Prefill-sized groups: LDS-DMA kernel, 256-column tiles of 256 / 128 / 64 rows.
template <int BN>
hipError_t launch_pair_dlds(const void* x_perm, const int32_t* expert_offsets, int cap_rows, int n_local, int H,
                            int I_s, const void* w_gate, const void* w_up, const void* w_down, void* h_ws,
                            void* y_perm, uint32_t flags, hipStream_t stream) {
  const bool y_bf16 = (flags & MOE_Y_PERM_BF16) != 0;
  const int m_blocks = gg::max_row_blocks(cap_rows, n_local);
  const dim3 block(256);
  const uint16_t* xp = static_cast<const uint16_t*>(x_perm);
  uint16_t* hw = static_cast<uint16_t*>(h_ws);
  auto grid_for = [&](int ncb) { return dim3((unsigned)((ncb * m_blocks + gg::kNumXcd - 1) / gg::kNumXcd * gg::kNumXcd)); };
  if (!(flags & MOE_FFN_SKIP_GATEUP)) {
    const int ncb = (I_s + BN / 2 - 1) / (BN / 2);
    hipLaunchKernelGGL((gg::grouped_gemm_dlds_kernel<BN, true, uint16_t>), grid_for(ncb), block, 0, stream, xp,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_gate),
                       static_cast<const uint16_t*>(w_up), I_s, H, hw, ncb);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
  }
  if (flags & MOE_FFN_SKIP_DOWN) return hipSuccess;
  const int ncb = (H + BN - 1) / BN;
  if (y_bf16)
    hipLaunchKernelGGL((gg::grouped_gemm_dlds_kernel<BN, false, uint16_t>), grid_for(ncb), block, 0, stream, hw,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_down),
                       static_cast<const uint16_t*>(nullptr), H, I_s, static_cast<uint16_t*>(y_perm), ncb);
  else
    hipLaunchKernelGGL((gg::grouped_gemm_dlds_kernel<BN, false, float>), grid_for(ncb), block, 0, stream, hw,
                       expert_offsets, n_local, cap_rows, static_cast<const uint16_t*>(w_down),
                       static_cast<const uint16_t*>(nullptr), H, I_s, static_cast<float*>(y_perm), ncb);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_expert_ffn(const void* x_perm, const int32_t* expert_offsets, int cap_rows, int n_local, int H,
                             int I_s, const void* w_gate, const void* w_up, const void* w_down, void* h_ws,
                             void* y_perm, uint32_t flags, hipStream_t stream) {
  if (cap_rows == 0) return hipSuccess;
  // Average rows per local expert decides the tile height: large groups take the 256x256
  // LDS-DMA kernel, small ones the 128x128 register-staged kernel.
  if (cap_rows / n_local >= 48)
    return launch_pair_dlds<256>(x_perm, expert_offsets, cap_rows, n_local, H, I_s, w_gate, w_up, w_down,
                                            h_ws, y_perm, flags, stream);
  return launch_pair<128, 128, 2, 2>(x_perm, expert_offsets, cap_rows, n_local, H, I_s, w_gate, w_up, w_down, h_ws,
                                     y_perm, flags, stream);
}

}  // namespace moe
