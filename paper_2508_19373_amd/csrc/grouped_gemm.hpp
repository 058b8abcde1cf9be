// Grouped "NT" GEMM for the expert networks, prefill-sized groups (gfx950).
//
//   C[r, n] = sum_k A[r, k] * B_e[n, k]      for the rows r of expert e (bf16 in, fp32 accumulate)
//
// GATEUP mode fuses the SwiGLU epilogue: the B tile interleaves 32-row blocks of the gate and
// up matrices of the same output columns, so the two accumulators a lane needs for
// silu(g) * u sit in the same lane and the activation never leaves registers.
//
// Design for CDNA4:
//  * one workgroup per (expert, row block, column block) tile; v_mfma_f32_32x32x16_bf16;
//  * operands go global -> LDS directly (global_load_lds_dwordx4, no VGPR staging), two LDS
//    stages of BM x 64 + BN x 64 bf16;
//  * LDS rows are 128 bytes; the 16-byte chunk index is XOR-swizzled with (row/2)%8, applied
//    on the global side of the DMA (a lane fetches the chunk that belongs at its LDS slot),
//    so operand reads (ds_read_b128) are bank-conflict free;
//  * one barrier per k-tile, placed after the last operand read of the tile, so the refill
//    of the stage just consumed and the first operand reads of the next tile overlap with the
//    last quarter of the tile's MFMAs;
//  * tile ids are remapped so that each of the 8 XCDs (which get workgroups round-robin) works
//    on a contiguous run of tiles that share A and B panels in its own L2.
#pragma once
#include <type_traits>

#include "moe_internal.hpp"

namespace moe {
namespace gg {

constexpr int BK = 64;          // K elements per LDS row (128 bytes, 8 chunks of 16 bytes)
constexpr int kNumXcd = 8;

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * BK + ((chunk ^ swz(row)) << 3); }
__device__ __forceinline__ int acc_row(int i, int lane) { return ((i >> 2) << 3) + ((lane >> 5) << 2) + (i & 3); }
__device__ __forceinline__ float silu_mul(float g, float u) { return g / (1.f + __expf(-g)) * u; }

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

// Row blocks of one expert: as many 256-row blocks as fit, then the remainder r is covered by
// the cheapest of {64}, {128}, {128 + 64}, {256} rows, so the padding per expert is below 64
// rows (padded rows are pure loss: only algorithmic FLOPs count).
struct RowBlocks {
  int n256, n128, n64;
  __device__ __forceinline__ int total() const { return n256 + n128 + n64; }
};
__device__ __forceinline__ RowBlocks row_blocks(int rows) {
  RowBlocks rb;
  const int r = rows & 255;
  rb.n256 = (rows >> 8) + (r > 192 ? 1 : 0);
  rb.n128 = (r > 64 && r <= 192) ? 1 : 0;
  rb.n64 = ((r > 0 && r <= 64) || (r > 128 && r <= 192)) ? 1 : 0;
  return rb;
}
// Host-side upper bound on sum_e row_blocks(rows_e).total() given sum_e rows_e <= cap_rows.
inline int max_row_blocks(int cap_rows, int n_local) { return cap_rows / 256 + 2 * n_local; }

struct TileCoord {
  int expert, row0, row_end, nb, height;  // height: 256, 128 or 64
  bool valid;
};

// Tile `lid` of the list: experts in order, inside an expert column blocks in order, inside a
// column block the row blocks (row block fastest, so neighbours share the B panel and a run of
// tiles covers all row blocks of a few column blocks).
__device__ __forceinline__ TileCoord find_tile(const int32_t* __restrict__ expert_offsets, int n_local,
                                               int n_col_blocks, int bid) {
  TileCoord t;
  t.valid = false;
  int total = 0;
  for (int e = 0; e < n_local; ++e)
    total += row_blocks(expert_offsets[e + 1] - expert_offsets[e]).total() * n_col_blocks;
  // XCD remap: workgroup b runs on XCD b % 8; give XCD x the tiles [x*chunk, (x+1)*chunk)
  const int chunk = (total + kNumXcd - 1) / kNumXcd;
  const int xcd = bid % kNumXcd, slot = bid / kNumXcd;
  if (slot >= chunk) return t;
  int lid = xcd * chunk + slot;
  if (lid >= total) return t;
  for (int e = 0; e < n_local; ++e) {
    const int lo = expert_offsets[e], hi = expert_offsets[e + 1];
    const RowBlocks rb = row_blocks(hi - lo);
    const int mbs = rb.total();
    const int tiles = mbs * n_col_blocks;
    if (lid < tiles) {
      const int mi = lid % mbs;
      t.expert = e;
      t.nb = lid / mbs;
      t.row_end = hi;
      if (mi < rb.n256) {
        t.height = 256;
        t.row0 = lo + mi * 256;
      } else if (mi < rb.n256 + rb.n128) {
        t.height = 128;
        t.row0 = lo + rb.n256 * 256;
      } else {
        t.height = 64;
        t.row0 = lo + rb.n256 * 256 + rb.n128 * 128;
      }
      t.valid = true;
      return t;
    }
    lid -= tiles;
  }
  return t;
}

// One (BM x BN) output tile, computed by the whole workgroup of WM x WN wavefronts.
template <int BM, int BN, int WM, int WN, bool GATEUP, typename OutT>
__device__ __forceinline__ void gemm_tile(uint16_t* smem, const TileCoord& tc, const uint16_t* __restrict__ A,
                                          int cap_rows, const uint16_t* __restrict__ B0,
                                          const uint16_t* __restrict__ B1, int n_out, int K,
                                          OutT* __restrict__ C) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
  constexpr int A_INST = BM / 8 / NW, B_INST = BN / 8 / NW;  // DMA instructions per wave per k-tile
  constexpr int NCOLS = GATEUP ? BN / 2 : BN;
  constexpr int STAGE = (BM + BN) * BK;  // uint16 elements per stage
  static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "tile / wave grid mismatch");
  static_assert((BM / 8) % NW == 0 && (BN / 8) % NW == 0, "loader mismatch");
  static_assert(!GATEUP || (TN % 2 == 0), "gate and up column blocks must pair up inside a wave");
  const int row0 = tc.row0, hi = tc.row_end, col0 = tc.nb * NCOLS;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // ---- DMA addressing: instruction `inst` fills LDS rows [8*inst, 8*inst+8); lane -> row
  // 8*inst + lane/8, physical chunk lane%8, which must hold logical chunk (lane%8) ^ swz(row).
  const uint16_t* a_src[A_INST];
  const uint16_t* b_src[B_INST];
#pragma unroll
  for (int j = 0; j < A_INST; ++j) {
    const int inst = j * NW + wave;
    const int r = inst * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz(r);
    const int gr = min(row0 + r, cap_rows - 1);  // rows past the group are fetched, never stored
    a_src[j] = A + (size_t)gr * K + c * 8;
  }
  const size_t expert_stride = (size_t)n_out * K;
#pragma unroll
  for (int j = 0; j < B_INST; ++j) {
    const int inst = j * NW + wave;
    const int r = inst * 8 + (lane >> 3);
    const int c = (lane & 7) ^ swz(r);
    const uint16_t* base = B0;
    int wrow;
    if (GATEUP) {  // 32-row blocks alternate gate, up, gate, up ... of the same output columns
      const int jb = r >> 5;
      wrow = col0 + (jb >> 1) * 32 + (r & 31);
      if (jb & 1) base = B1;
    } else {
      wrow = col0 + r;
    }
    wrow = min(wrow, n_out - 1);
    b_src[j] = base + (size_t)tc.expert * expert_stride + (size_t)wrow * K + c * 8;
  }

  // DMA instruction `idx` of a k-tile: the B (weight) rows first -- they come from HBM for the
  // first time and need the longest flight -- then the A rows, which are re-read by every column
  // block and mostly hit in L2.
  constexpr int N_DMA = A_INST + B_INST;
  auto issue_dma = [&](int kt, int stage, auto idx_tag) {
    constexpr int idx = decltype(idx_tag)::value;
    uint16_t* sa = smem + stage * STAGE;
    uint16_t* sb = sa + BM * BK;
    if constexpr (idx < B_INST) {
      __builtin_amdgcn_global_load_lds((global_void_t*)(b_src[idx] + (size_t)kt * BK),
                                       (lds_void_t*)(sb + (idx * NW + wave) * 8 * BK), 16, 0, 0);
    } else {
      constexpr int j = idx - B_INST;
      __builtin_amdgcn_global_load_lds((global_void_t*)(a_src[j] + (size_t)kt * BK),
                                       (lds_void_t*)(sa + (j * NW + wave) * 8 * BK), 16, 0, 0);
    }
  };

  const int a_row = wm * (BM / WM) + (lane & 31);
  const int b_row = wn * (BN / WN) + (lane & 31);
  const int kq = lane >> 5;
  // operand `r` of a k16 step: r < TM is the A fragment of row block r, else a B fragment
  auto read_frag = [&](int stage, int ks, auto r_tag, bf16x8(&af)[TM], bf16x8(&bfr)[TN]) {
    constexpr int r = decltype(r_tag)::value;
    const uint16_t* sa = smem + stage * STAGE;
    const uint16_t* sb = sa + BM * BK;
    const int c = ks * 2 + kq;
    if constexpr (r < TM)
      af[r] = *reinterpret_cast<const bf16x8*>(sa + lds_off(a_row + r * 32, c));
    else
      bfr[r - TM] = *reinterpret_cast<const bf16x8*>(sb + lds_off(b_row + (r - TM) * 32, c));
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk = K / BK;
  bf16x8 af0[TM], bf0[TN], af1[TM], bf1[TN];
  constexpr int NM = TM * TN, NDS = TM + TN;
  constexpr int RD_SLOTS = NM * 3 / 4;

  // One k16 step in a fixed instruction order: the NM MFMAs on the operands (af, bfr), and
  // between them, evenly spread, (READS) the NDS reads of the next step's operands into (afn,
  // bfn) from LDS stage rd_stage / step rd_ks, and the DMA instructions [DLO, DHI) of k-tile
  // dma_kt into LDS stage dma_stage.  Each MFMA and the memory instructions that follow it are
  // fenced, so the matrix pipe never waits behind a burst of memory instructions and the
  // texture-address unit sees a steady stream of DMA requests that it can accept without
  // stalling the wave.
  auto k_step = [&](const bf16x8(&af)[TM], const bf16x8(&bfr)[TN], auto reads_tag, int rd_stage, int rd_ks,
                    bf16x8(&afn)[TM], bf16x8(&bfn)[TN], auto dlo_tag, auto dhi_tag, int dma_kt, int dma_stage) {
    constexpr bool READS = decltype(reads_tag)::value;
    constexpr int DLO = decltype(dlo_tag)::value, NVM = decltype(dhi_tag)::value - DLO;
    static_for<0, NM>([&](auto m_tag) {
      constexpr int m = decltype(m_tag)::value;
      constexpr int i = m / TN, j = m % TN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      if constexpr (READS && m < RD_SLOTS) {  // operand reads finish early in the step
        static_for<(m * NDS) / RD_SLOTS, ((m + 1) * NDS) / RD_SLOTS>(
            [&](auto r_tag) { read_frag(rd_stage, rd_ks, r_tag, afn, bfn); });
      }
      static_for<DLO + (m * NVM) / NM, DLO + ((m + 1) * NVM) / NM>(
          [&](auto d_tag) { issue_dma(dma_kt, dma_stage, d_tag); });
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // The DMA of a k-tile is issued in three slices over the three k16 steps that follow the
  // release of its LDS stage; the fourth step gives the last slice time to land.
  constexpr int D0 = (N_DMA * 3 + 7) / 8;        // right after the barrier (step 3 of tile kt)
  constexpr int D1 = D0 + (N_DMA - D0 + 1) / 2;  // step 0 of tile kt+1; the rest in step 1
  using T_ = std::true_type;
  using F_ = std::false_type;
  template_int<0> i0_;
  template_int<D0> iD0_;
  template_int<D1> iD1_;
  template_int<N_DMA> iN_;

  // One k-tile.  L01: issue the rest of tile kt+1's DMA during steps 0 and 1.  SYNC: after the
  // tile's last operand read, wait for tile kt+1, barrier, then (L3) start refilling the stage
  // just consumed with tile kt+2 and prefetch tile kt+1's first operands, all overlapped with
  // the last quarter of this tile's MFMAs.
  auto k_tile = [&](int kt, auto l01_tag, auto sync_tag, auto l3_tag) {
    constexpr bool L01 = decltype(l01_tag)::value, SYNC = decltype(sync_tag)::value, L3 = decltype(l3_tag)::value;
    const int cur = kt & 1;
    if constexpr (L01) {
      k_step(af0, bf0, T_{}, cur, 1, af1, bf1, iD0_, iD1_, kt + 1, cur ^ 1);
      k_step(af1, bf1, T_{}, cur, 2, af0, bf0, iD1_, iN_, kt + 1, cur ^ 1);
    } else {
      k_step(af0, bf0, T_{}, cur, 1, af1, bf1, i0_, i0_, 0, 0);
      k_step(af1, bf1, T_{}, cur, 2, af0, bf0, i0_, i0_, 0, 0);
    }
    k_step(af0, bf0, T_{}, cur, 3, af1, bf1, i0_, i0_, 0, 0);
    if constexpr (SYNC) {
      wait_lgkmcnt0();  // my reads of stage `cur` are done
      wait_vmcnt<0>();  // tile kt+1 has landed in the other stage
      __builtin_amdgcn_s_barrier();
      if constexpr (L3)
        k_step(af1, bf1, T_{}, cur ^ 1, 0, af0, bf0, i0_, iD0_, kt + 2, cur);
      else
        k_step(af1, bf1, T_{}, cur ^ 1, 0, af0, bf0, i0_, i0_, 0, 0);
    } else {
      k_step(af1, bf1, F_{}, 0, 0, af0, bf0, i0_, i0_, 0, 0);
    }
  };

  static_for<0, N_DMA>([&](auto d_tag) { issue_dma(0, 0, d_tag); });
  wait_vmcnt<0>();
  __builtin_amdgcn_s_barrier();
  if (nk > 1) static_for<0, D0>([&](auto d_tag) { issue_dma(1, 1, d_tag); });
  static_for<0, NDS>([&](auto r_tag) { read_frag(0, 0, r_tag, af0, bf0); });
  for (int kt = 0; kt + 2 < nk; ++kt) k_tile(kt, T_{}, T_{}, T_{});
  if (nk > 1) k_tile(nk - 2, T_{}, T_{}, F_{});
  k_tile(nk - 1, F_{}, F_{}, F_{});

  // ---- epilogue
  const int lcol = lane & 31;
  const bool full = (row0 + BM <= hi) && (col0 + NCOLS <= n_out);
  auto store_tile = [&](auto guard) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int rbase = row0 + wm * (BM / WM) + i * 32;
      if constexpr (GATEUP) {
#pragma unroll
        for (int j = 0; j < TN; j += 2) {
          const int jb = wn * TN + j;  // even: gate block; jb + 1: up block of the same columns
          const int col = col0 + (jb >> 1) * 32 + lcol;
          uint16_t* cp = reinterpret_cast<uint16_t*>(C) + (size_t)rbase * n_out + col;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int ro = acc_row(v, lane);
            if (guard(rbase + ro, col))
              cp[(size_t)ro * n_out] = (uint16_t)f32_to_bf16_bits(silu_mul(acc[i][j][v], acc[i][j + 1][v]));
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = col0 + wn * (BN / WN) + j * 32 + lcol;
          OutT* cp = C + (size_t)rbase * n_out + col;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int ro = acc_row(v, lane);
            if (guard(rbase + ro, col)) {
              if constexpr (sizeof(OutT) == 4)
                cp[(size_t)ro * n_out] = acc[i][j][v];
              else
                cp[(size_t)ro * n_out] = (OutT)f32_to_bf16_bits(acc[i][j][v]);
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

// Kernel: 256 threads (4 wavefronts); each workgroup computes one tile of the list, whose
// height (256, 128 or 64 rows) selects the wave arrangement.
template <int BN, bool GATEUP, typename OutT>
__global__ __launch_bounds__(256) void grouped_gemm_dlds_kernel(
    const uint16_t* __restrict__ A, const int32_t* __restrict__ expert_offsets, int n_local, int cap_rows,
    const uint16_t* __restrict__ B0, const uint16_t* __restrict__ B1, int n_out, int K, OutT* __restrict__ C,
    int n_col_blocks) {
  __shared__ __attribute__((aligned(1024))) uint16_t smem[2 * (256 + BN) * BK];
  const TileCoord tc = find_tile(expert_offsets, n_local, n_col_blocks, blockIdx.x);
  if (!tc.valid) return;
  if (tc.height == 256)
    gemm_tile<256, BN, 2, 2, GATEUP, OutT>(smem, tc, A, cap_rows, B0, B1, n_out, K, C);
  else if (tc.height == 128)
    gemm_tile<128, BN, 2, 2, GATEUP, OutT>(smem, tc, A, cap_rows, B0, B1, n_out, K, C);
  else
    gemm_tile<64, BN, 1, 4, GATEUP, OutT>(smem, tc, A, cap_rows, B0, B1, n_out, K, C);
}

}  // namespace gg
}  // namespace moe
