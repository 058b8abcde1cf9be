// Grouped "NT" GEMM for the expert networks, prefill-sized groups (gfx950).
//
//   C[r, n] = sum_k A[r, k] * B_e[n, k]      for the rows r of expert e (bf16 in, fp32 accumulate)
//
// GATEUP mode fuses the SwiGLU epilogue: the B tile interleaves 32-row blocks of the gate and
// up matrices of the same output columns, so the two accumulators a lane needs for
// silu(g) * u sit in the same lane and the activation never leaves registers.
//
// Design for CDNA4:
//  * one workgroup per (expert, row block, column block) tile, 4 wavefronts of 128 x 128 outputs;
//  * operands go global -> LDS directly (global_load_lds_dwordx4, no VGPR staging) into all
//    160 KB of LDS: 2 activation + 3 weight stages of a 64-wide k-tile for a 256-row tile, 3 + 3 and
//    4 + 4 stages for the 128- and 64-row remainder tiles (an HBM round trip under load is longer
//    than one k-tile of MFMA work);
//  * LDS rows are 128 bytes; the 16-byte chunk index is XOR-swizzled with (row/2)%8, applied
//    on the global side of the DMA (a lane fetches the chunk that belongs at its LDS slot),
//    so operand reads (ds_read_b128) are bank-conflict free;
//  * v_mfma_f32_16x16x32_bf16 in back-to-back pairs on one accumulator, operands of the whole
//    k-tile resident in registers and refreshed in place (see gemm_tile): the chip is power
//    limited, and this instruction mix sustains the most FLOP/s at the cap;
//  * one barrier per k-tile; DMA issue and operand reads are spread between the MFMA pairs in a
//    fixed, fenced order (a burst of DMA instructions stalls the wave on the address unit);
//  * tile ids are remapped so that each of the 8 XCDs (which get workgroups round-robin) works
//    on a contiguous run of tiles that share A and B panels in its own L2; remainder tiles run
//    after all full tiles, so concurrent full tiles stay in k-lockstep (see find_unit).
#pragma once
#include <cmath>
#include <type_traits>

#include "moe_internal.hpp"
#include "unit_list_even.hpp"
#include "unit_list_wave.hpp"

namespace moe {
namespace gg {

constexpr int BK = 64;          // K elements per LDS row (128 bytes, 8 chunks of 16 bytes)

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * BK + ((chunk ^ swz(row)) << 3); }
__device__ __forceinline__ float silu_mul(float g, float u) { return g * __builtin_amdgcn_rcpf(1.f + __expf(-g)) * u; }

// s_waitcnt with only vmcnt / only lgkmcnt constrained (gfx9 encoding)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }


template <int N>
using template_int = std::integral_constant<int, N>;

// Compile-time loop: f(std::integral_constant<int, I>{}) for I in [LO, HI).
template <int LO, int HI, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (LO < HI) {
    f(std::integral_constant<int, LO>{});
    static_for<LO + 1, HI>(f);
  }
}

constexpr int kLdsBytes = 160 * 1024;

// DMA bookkeeping of gemm_tile.  Tile t issues, in this order, the activation loads of tile t+NSA
// (A_INST instructions, if that tile exists) and the weight loads of tile t+NSB (B_INST, likewise).
// Loads complete in issue order, so at the barrier of the tile that has `j` tiles after it, the
// loads that may stay in flight are those issued after the youngest one the next tile needs.
constexpr int dma_slack(int j, int NSA, int NSB, int A_INST, int B_INST) {
  int n = 0;
  // the next tile's activations were issued NSA-1 tiles ago; the weights of that group are younger
  if (NSA < NSB && j - 1 + NSA >= NSB) n += B_INST;
  for (int jt = j + NSA - 2; jt >= j + 1; --jt)  // whole groups of the tiles in between
    n += (jt >= NSA ? A_INST : 0) + (jt >= NSB ? B_INST : 0);
  return n;
}

// One (BM x BN) output tile, computed by the whole workgroup of WM x WN wavefronts, on
// v_mfma_f32_16x16x32_bf16 with the k-tile's operands resident in registers.
//
// MI355X is power-limited under dense MFMA load, and pairs of 16x16x32 MFMAs issued back to back
// on the same accumulator sustain ~12 % more FLOP/s at the power cap than 32x32x16 (they move
// half the accumulator bytes per FLOP).  Pairing needs both k32 halves of a 64-wide k-tile for
// the same accumulator, so the operands of the WHOLE k-tile live in registers (2*(TM+TN)
// fragments) and are refreshed in place: a fragment is re-read from the next k-tile's LDS stage
// right after its last use.  LDS is then a multi-stage landing buffer in front of the register
// tile, still with one barrier per k-tile.
// The traversal order and the refresh schedule are described at k_tile below.
template <int BM, int BN, int WM, int WN, int NSA, int NSB, bool GATEUP, typename OutT>
__device__ __forceinline__ void gemm_tile(uint16_t* smem, const TileCoord& tc, const uint16_t* __restrict__ A,
                                            int cap_rows, const uint16_t* __restrict__ B0,
                                            const uint16_t* __restrict__ B1, int n_out, int K, int kt0, int nk,
                                            OutT* __restrict__ C, const RowMap rows = RowMap{nullptr, 1}) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 16, TN = BN / WN / 16;
  constexpr int A_INST = BM / 8 / NW, B_INST = BN / 8 / NW;
  constexpr int NCOLS = GATEUP ? BN / 2 : BN;
  constexpr int A_STAGE = BM * BK, B_STAGE = BN * BK;  // LDS: NSA activation stages, then NSB weight stages
  static_assert(NSA >= 2 && NSA <= NSB, "activations need at least two stages and no more than the weights");
  static_assert((NSA * A_STAGE + NSB * B_STAGE) * 2 <= kLdsBytes, "LDS budget");
  constexpr int NP = TM * TN;  // MFMA pairs per k-tile
  static_assert(BM % (WM * 16) == 0 && BN % (WN * 16) == 0, "tile / wave grid mismatch");
  static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "loader mismatch");
  static_assert(!GATEUP || (TN % 2 == 0), "gate and up column blocks must pair up inside a wave");
  static_assert(TM >= 3, "needs a first, a middle and a last row block");
  const int row0 = tc.row0, hi = tc.row_end, col0 = tc.nb * NCOLS;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  const uint16_t* a_src[A_INST];
  const uint16_t* b_src[B_INST];
#pragma unroll
  for (int j = 0; j < A_INST; ++j) {
    const int inst = j * NW + wave;
    const int r = inst * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz(r);
    // rows past the tile's expert are computed and dropped: they read any valid row (with a row
    // map, the expert's last one: entries past the routed rows are not defined)
    const int gr = rows.row_src ? rows(min(row0 + r, hi - 1)) : min(row0 + r, cap_rows - 1);
    a_src[j] = A + (size_t)gr * K + (size_t)kt0 * BK + c * 8;
  }
  const size_t expert_stride = (size_t)n_out * K;
#pragma unroll
  for (int j = 0; j < B_INST; ++j) {
    const int inst = j * NW + wave;
    const int r = inst * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz(r);
    const uint16_t* base = B0;
    int wrow;
    if (GATEUP) {  // 16-row blocks alternate gate, up, gate, up ... of the same output columns
      const int jb = r >> 4;
      wrow = col0 + (jb >> 1) * 16 + (r & 15);
      if (jb & 1) base = B1;
    } else {
      wrow = col0 + r;
    }
    wrow = min(wrow, n_out - 1);
    b_src[j] = base + (size_t)tc.expert * expert_stride + (size_t)wrow * K + (size_t)kt0 * BK + c * 8;
  }

  constexpr int N_DMA = A_INST + B_INST;
  // DMA instruction `idx` of a k-tile's group: the activation rows first, then the weight rows
  // (loads complete in issue order, and the activations are the operand needed soonest)
  auto issue_dma = [&](int kt_a, int stage_a, int kt_b, int stage_b, auto idx_tag) {
    constexpr int idx = decltype(idx_tag)::value;
    if constexpr (idx < A_INST) {
      __builtin_amdgcn_global_load_lds((global_void_t*)(a_src[idx] + (size_t)kt_a * BK),
                                       (lds_void_t*)(smem + stage_a * A_STAGE + (idx * NW + wave) * 8 * BK), 16, 0, 0);
    } else {
      constexpr int j = idx - A_INST;
      __builtin_amdgcn_global_load_lds(
          (global_void_t*)(b_src[j] + (size_t)kt_b * BK),
          (lds_void_t*)(smem + NSA * A_STAGE + stage_b * B_STAGE + (j * NW + wave) * 8 * BK), 16, 0, 0);
    }
  };

  const int a_row = wm * (BM / WM) + (lane & 15);
  const int b_row = wn * (BN / WN) + (lane & 15);
  const int kq = lane >> 4;
  bf16x8 af[TM][2], bfr[TN][2];
  auto read_a = [&](int stage, auto i_tag, auto ks_tag) {
    constexpr int i = decltype(i_tag)::value, ks = decltype(ks_tag)::value;
    af[i][ks] = *reinterpret_cast<const bf16x8*>(smem + stage * A_STAGE + lds_off(a_row + i * 16, ks * 4 + kq));
  };
  auto read_b = [&](int stage, auto j_tag, auto ks_tag) {
    constexpr int j = decltype(j_tag)::value, ks = decltype(ks_tag)::value;
    bfr[j][ks] = *reinterpret_cast<const bf16x8*>(smem + NSA * A_STAGE + stage * B_STAGE +
                                                  lds_off(b_row + j * 16, ks * 4 + kq));
  };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  using T_ = std::true_type;
  using F_ = std::false_type;
  template_int<0> k0_;
  template_int<1> k1_;
  // DMA instruction d of a group goes after pair TN + d * DSPAN / (group size): spread over the
  // whole tile after the barrier (a burst of DMA instructions stalls the wave on the address unit)
  constexpr int DSPAN = NP - TN;

  // One k-tile with `sa`, `sb` the LDS stages that hold its activations and weights.
  // SYNC: barrier after the first row, then refresh the register operands from the next stages.
  // DMA_A / DMA_B: refill this tile's stages with the activations of tile kt+NSA / the weights of
  // tile kt+NSB, one instruction every few pairs.  SLACK: DMA instructions that may still be in
  // flight at the barrier (those issued after the ones tile kt+1 needs; loads complete in order).
  // Pair order: the upper half of the row blocks row by row, the lower half column by column, so
  // operand fragments die -- and are refreshed -- at an even pace (at most 2 LDS reads per pair;
  // reading all B fragments in the last row made that row LDS-bound):
  //   pair p < TM            : A[TM/2 + p/2][p%2] of THIS tile (lower-half A rows die at the tile's end);
  //                            these TM reads must be issued before the barrier behind pair TN - 1 (the
  //                            stage is refilled after it), so with TM > TN they are dealt over the
  //                            first TN pairs
  //   end of upper row i     : A[i] of the next tile
  //   end of lower column j  : B[j] of the next tile
  constexpr int HM = TM / 2, NP1 = HM * TN;
  static_assert(TM % 2 == 0, "pair order needs an even row-block count");
  constexpr int LOWER_SPAN = TM <= TN ? TM : TN;  // pairs over which the lower-half reads are dealt
  auto k_tile = [&](int kt, int sa, int sb, auto sync_tag, auto dma_a_tag, auto dma_b_tag, auto slack_tag) {
    constexpr bool SYNC = decltype(sync_tag)::value;
    constexpr bool DMA_A = decltype(dma_a_tag)::value, DMA_B = decltype(dma_b_tag)::value;
    constexpr int SLACK = decltype(slack_tag)::value;
    constexpr int ND = DMA_B ? N_DMA : (DMA_A ? A_INST : 0);
    static_assert(DMA_A || !DMA_B, "weights are prefetched at least as deep as activations");
    const int sa_n = (sa + 1 == NSA) ? 0 : sa + 1, sb_n = (sb + 1 == NSB) ? 0 : sb + 1;
    static_for<0, NP>([&](auto p_tag) {
      constexpr int p = decltype(p_tag)::value;
      constexpr bool upper = p < NP1;
      constexpr int i = upper ? p / TN : HM + (p - NP1) % HM;
      constexpr int j = upper ? p % TN : (p - NP1) / HM;
      // weights as the MFMA "A" operand, activations as "B": the result tile is the transpose, so a
      // lane ends up with 4 CONSECUTIVE output columns of one row (one 8- or 16-byte store)
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j][0], af[i][0], acc[i][j], 0, 0, 0);
      acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[j][1], af[i][1], acc[i][j], 0, 0, 0);
      if constexpr (p < LOWER_SPAN)
        static_for<(p * TM + LOWER_SPAN - 1) / LOWER_SPAN, ((p + 1) * TM + LOWER_SPAN - 1) / LOWER_SPAN>([&](auto r_tag) {
          constexpr int r = decltype(r_tag)::value;
          read_a(sa, template_int<HM + r / 2>{}, template_int<r % 2>{});
        });
      if constexpr (SYNC) {
        if constexpr (upper && j == TN - 1 && p >= TN) {  // rows 1..HM-1: after the barrier
          read_a(sa_n, template_int<i>{}, k0_);
          read_a(sa_n, template_int<i>{}, k1_);
        }
        if constexpr (p == TN + 1) {  // row 0 died before the barrier: refresh it right after
          read_a(sa_n, template_int<0>{}, k0_);
          read_a(sa_n, template_int<0>{}, k1_);
        }
        if constexpr (!upper && i == TM - 1) {
          read_b(sb_n, template_int<j>{}, k0_);
          read_b(sb_n, template_int<j>{}, k1_);
        }
      }
      if constexpr (ND > 0 && p >= TN && p < TN + DSPAN) {
        constexpr int q = p - TN;
        static_for<(q * ND) / DSPAN, ((q + 1) * ND) / DSPAN>(
            [&](auto d_tag) { issue_dma(kt + NSA, sa, kt + NSB, sb, d_tag); });
      }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (SYNC && p == TN - 1) {
        wait_lgkmcnt0();       // my reads of this tile's activation stage are done
        wait_vmcnt<SLACK>();   // tile kt+1 has landed
        __builtin_amdgcn_s_barrier();
      }
    });
  };
  auto next_a = [](int st) { return (st + 1 == NSA) ? 0 : st + 1; };
  auto next_b = [](int st) { return (st + 1 == NSB) ? 0 : st + 1; };

  // prologue: tile 0, then the groups that tiles -(NSB-1) .. -1 would have issued, in their order
  static_for<0, N_DMA>([&](auto d_tag) { issue_dma(0, 0, 0, 0, d_tag); });
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  static_for<1 - NSB, 0>([&](auto t_tag) {
    constexpr int t = decltype(t_tag)::value;
    if constexpr (t + NSA > 0) {
      if (t + NSA < nk) static_for<0, A_INST>([&](auto d_tag) { issue_dma(t + NSA, t + NSA, 0, 0, d_tag); });
    }
    if (t + NSB < nk) static_for<A_INST, N_DMA>([&](auto d_tag) { issue_dma(0, 0, t + NSB, t + NSB, d_tag); });
  });
  static_for<0, TM>([&](auto i_tag) {
    read_a(0, i_tag, k0_);
    read_a(0, i_tag, k1_);
  });
  static_for<0, TN>([&](auto j_tag) {
    read_b(0, j_tag, k0_);
    read_b(0, j_tag, k1_);
  });
  int sa = 0, sb = 0, kt = 0;
  for (; kt + NSB < nk; ++kt) {  // steady state: both refills exist
    k_tile(kt, sa, sb, T_{}, T_{}, T_{}, template_int<dma_slack(NSA + NSB, NSA, NSB, A_INST, B_INST)>{});
    sa = next_a(sa);
    sb = next_b(sb);
  }
  static_for<0, NSB - 1>([&](auto q_tag) {  // the last tiles but one: j tiles follow, no weight refill left
    constexpr int j = NSB - 1 - decltype(q_tag)::value;
    if (nk - 1 - j >= 0) {
      k_tile(nk - 1 - j, sa, sb, T_{}, std::integral_constant<bool, (j >= NSA)>{}, F_{},
             template_int<dma_slack(j, NSA, NSB, A_INST, B_INST)>{});
      sa = next_a(sa);
      sb = next_b(sb);
    }
  });
  k_tile(nk - 1, sa, sb, F_{}, F_{}, F_{}, template_int<0>{});

  // ---- epilogue: accumulator register v of tile (i, j) is row i*16 + lane%16, column
  // j*16 + (lane/16)*4 + v of the wave's sub-tile
  const int lrow = lane & 15, lcol = (lane >> 4) * 4;
  const bool full = (row0 + BM <= hi) && (col0 + NCOLS <= n_out);  // n_out is a multiple of 4
  auto store_tile = [&](auto guard) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = row0 + wm * (BM / WM) + i * 16 + lrow;
      if constexpr (GATEUP) {
#pragma unroll
        for (int j = 0; j < TN; j += 2) {
          const int jb = wn * TN + j;  // even: gate block; jb + 1: up block of the same columns
          const int col = col0 + (jb >> 1) * 16 + lcol;
          if (guard(row, col)) {
            uint2 o;
            o.x = pack_bf16x2(silu_mul(acc[i][j][0], acc[i][j + 1][0]), silu_mul(acc[i][j][1], acc[i][j + 1][1]));
            o.y = pack_bf16x2(silu_mul(acc[i][j][2], acc[i][j + 1][2]), silu_mul(acc[i][j][3], acc[i][j + 1][3]));
            *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(C) + (size_t)row * n_out + col) = o;
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = col0 + wn * (BN / WN) + j * 16 + lcol;
          if (guard(row, col)) {
            if constexpr (sizeof(OutT) == 4) {
              *reinterpret_cast<float4*>(C + (size_t)row * n_out + col) =
                  make_float4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
            } else {
              uint2 o;
              o.x = pack_bf16x2(acc[i][j][0], acc[i][j][1]);
              o.y = pack_bf16x2(acc[i][j][2], acc[i][j][3]);
              *reinterpret_cast<uint2*>(C + (size_t)row * n_out + col) = o;
            }
          }
        }
      }
    }
  };
  if (full)
    store_tile([](int, int) { return true; });
  else
    store_tile([&](int row, int col) { return row < hi && col < n_out; });
}

// Kernel: 256 threads (4 wavefronts); each workgroup computes one tile, whose height class
// selects the wave arrangement and the LDS stage counts.  SLICED (fp32 down projection): tiles may
// be cut along K as choose_slices decides from the routing; slice 0 of a tile writes `y`, slice
// z >= 1 its partial sums into `C` (see sliced_rows), which sum_sliced_kernel adds to y.  A separate
// instantiation, so that the unsliced kernels keep their register allocation.
template <int BN, bool GATEUP, typename OutT, bool SLICED>
__global__ __launch_bounds__(256) void grouped_gemm_dlds_kernel(
    const uint16_t* __restrict__ A, const int32_t* __restrict__ expert_offsets, int n_local, int cap_rows,
    const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1, int n_out, int K, OutT* __restrict__ C,
    int n_col_blocks, OutT* __restrict__ y, int max_slices, const RowMap rows) {
  __shared__ __attribute__((aligned(1024))) uint16_t smem[kLdsBytes / 2];
  int nk = K / BK, kt0 = 0, cls;
  OutT* out = C;
  TileCoord tc;
  if constexpr (SLICED) {
    const WaveSlicedUnit u = find_sliced_unit_of(expert_offsets, n_local, n_col_blocks, nk, max_slices, blockIdx.x);
    if (!u.valid) return;
    if (u.cls == 3) {  // a whole tile: the same call as in the unsliced kernel, constants included
      gemm_tile<256, BN, 2, 2, 2, 3, GATEUP, OutT>(smem, u.tc, A, cap_rows, B0, B1, n_out, K, 0, K / BK, y);
      return;
    }
    cls = u.cls;
    tc = u.tc;
    kt0 = u.kt0;
    nk = u.nk;
    out = u.z == 0 ? y : C + u.scratch_shift * n_out;
  } else {
    if (!find_tile(expert_offsets, n_local, n_col_blocks, blockIdx.x, cls, tc)) return;
  }
  if (cls == 0)
    gemm_tile<256, BN, 2, 2, 2, 3, GATEUP, OutT>(smem, tc, A, cap_rows, B0, B1, n_out, K, kt0, nk, out, rows);
  else if (cls == 1)
    gemm_tile<128, BN, 2, 2, 3, 3, GATEUP, OutT>(smem, tc, A, cap_rows, B0, B1, n_out, K, kt0, nk, out, rows);
  else
    gemm_tile<64, BN, 1, 4, 4, 4, GATEUP, OutT>(smem, tc, A, cap_rows, B0, B1, n_out, K, kt0, nk, out, rows);
}

// The same GEMM on the work list of unit_list_even.hpp: every tile is 160 rows x 256 weight rows, four
// wavefronts side by side, each with all 160 rows and 64 weight rows (10 x 4 accumulator blocks), three
// LDS stages of each operand.  Chosen on the host for launches with a few hundred rows per expert.
template <int BN, bool GATEUP, typename OutT>
__global__ __launch_bounds__(256) void grouped_gemm_even_kernel(
    const uint16_t* __restrict__ A, const int32_t* __restrict__ expert_offsets, int n_local, int cap_rows,
    const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1, int n_out, int K, OutT* __restrict__ C,
    int n_col_blocks, const RowMap rows) {
  __shared__ __attribute__((aligned(1024))) uint16_t smem[kLdsBytes / 2];
  TileCoord tc;
  if (!even_find_tile(expert_offsets, n_local, n_col_blocks, blockIdx.x, tc)) return;
  gemm_tile<kEvenRows, BN, 1, 4, 3, 3, GATEUP, OutT>(smem, tc, A, cap_rows, B0, B1, n_out, K, 0, K / BK, C, rows);
}

// y[r, :] += partial sums of slices 1, 2, ... in that order, for the rows the sliced kernel cut
// along K (it repeats that kernel's decision).  A workgroup adds 1024 columns of one row at a time:
// grid.x walks the rows, grid.y the column chunks.
__global__ __launch_bounds__(256) void sum_sliced_kernel(const float* __restrict__ partial,
                                                        const int32_t* __restrict__ expert_offsets, int n_local,
                                                        int n_col_blocks, int nk, int max_slices, int n_out,
                                                        float* __restrict__ y) {
  const SumPlan plan = sum_plan(expert_offsets, n_local, n_col_blocks, nk, max_slices);
  if (plan.slices == 1) return;
  const int total = plan.total;
  const size_t stride = (size_t)total * n_out / 4;
  const float4* p = reinterpret_cast<const float4*>(partial);
  for (int i = blockIdx.x; i < total; i += gridDim.x) {
    const int row = sum_plan_row(plan, expert_offsets, n_local, i);
    float4* yr = reinterpret_cast<float4*>(y + (size_t)row * n_out);
    const float4* pr = p + (size_t)i * n_out / 4;
    for (int c = blockIdx.y * blockDim.x + threadIdx.x; c < n_out / 4; c += gridDim.y * blockDim.x) {
      // all loads first (one memory latency instead of one per slice), then the sum in slice order
      float4 v[kMaxKSlices - 1];
#pragma unroll
      for (int z = 1; z < kMaxKSlices; ++z)
        if (z < plan.slices) v[z - 1] = pr[(z - 1) * stride + c];
      float4 acc = yr[c];
#pragma unroll
      for (int z = 1; z < kMaxKSlices; ++z) {
        if (z < plan.slices) {
          acc.x += v[z - 1].x;
          acc.y += v[z - 1].y;
          acc.z += v[z - 1].z;
          acc.w += v[z - 1].w;
        }
      }
      yr[c] = acc;
    }
  }
}

}  // namespace gg
}  // namespace moe
