// Work list of the grouped GEMM with row blocks of one height (kEvenRows = 160 rows).
//
// With a few hundred rows per expert (Qwen1.5-MoE at 4096 tokens: 60 experts of 250 to 300 rows) the
// 256-row tiling gives most experts one 256-row tile and one 64-row remainder tile per column block,
// and the remainder tile streams the expert's weight panel from HBM a second time: the gate/up
// projection then moves 1.24 GB for 0.69 GB of weights and is bound by HBM, not by the matrix cores.
// Here every expert's rows are cut into ceil(rows / 160) blocks of 160 rows, all tiles have the same
// shape and duration, and the row blocks of one (expert, column block) are neighbours in the list, so
// they walk K in lockstep and the second reader of the weight panel finds it in its XCD's L2.
// One class of tiles only: the list is the experts in order, inside an expert the column blocks,
// inside a column block the row blocks; virtual workgroup ids are dealt to the XCDs as in
// unit_list.hpp (id b runs on XCD b % 8; each XCD takes a contiguous eighth of the list).
#pragma once
#include "unit_list_wave.hpp"

namespace moe {
namespace gg {

constexpr int kEvenRows = 160;

__host__ __device__ inline int even_blocks(int rows) { return (rows + kEvenRows - 1) / kEvenRows; }

__host__ __device__ inline int even_tiles(const int32_t* __restrict__ expert_offsets, int n_local, int n_col_blocks) {
  int blocks = 0;
  for (int e = 0; e < n_local; ++e) blocks += even_blocks(expert_offsets[e + 1] - expert_offsets[e]);
  return blocks * n_col_blocks;
}

// Tile index of virtual workgroup id `vb` among n_tiles, or -1.
__host__ __device__ inline int even_tile_index(int n_tiles, int vb) {
  const int chunk = (n_tiles + kNumXcd - 1) / kNumXcd;
  const int xcd = vb % kNumXcd, slot = vb / kNumXcd;
  if (slot >= chunk) return -1;
  const int idx = xcd * chunk + slot;
  return idx < n_tiles ? idx : -1;
}

__host__ __device__ inline TileCoord even_locate(const int32_t* __restrict__ expert_offsets, int n_local,
                                                 int n_col_blocks, int idx) {
  TileCoord t = {0, 0, 0, 0};
  for (int e = 0; e < n_local; ++e) {
    const int lo = expert_offsets[e], hi = expert_offsets[e + 1];
    const int mbs = even_blocks(hi - lo), tiles = mbs * n_col_blocks;
    if (idx < tiles) {
      t.expert = e;
      t.nb = idx / mbs;
      t.row0 = lo + (idx % mbs) * kEvenRows;
      t.row_end = hi;
      return t;
    }
    idx -= tiles;
  }
  return t;
}

// Host-side bound on the virtual ids for any routing with sum of rows <= cap_rows.
inline int even_max_ids(int cap_rows, int n_local, int n_col_blocks) {
  const int tiles = (cap_rows / kEvenRows + n_local) * n_col_blocks;
  return kNumXcd * ((tiles + kNumXcd - 1) / kNumXcd);
}

// The tile of virtual id `vb`, found by one wavefront (lane l holds experts l, l + 64, ...); plain
// loops for a handful of experts.  Returns false if the id holds no tile.
__device__ inline bool even_find_tile(const int32_t* __restrict__ expert_offsets, int n_local, int n_col_blocks,
                                      int vb, TileCoord& tc) {
  if (n_local <= kPlainLoopExperts) {
    const int idx = even_tile_index(even_tiles(expert_offsets, n_local, n_col_blocks), vb);
    if (idx < 0) return false;
    tc = even_locate(expert_offsets, n_local, n_col_blocks, idx);
    return true;
  }
  WaveRouting w;
  const int lane = threadIdx.x & 63;
  w.chunks = (n_local + 63) >> 6;
  int mbs[kLaneChunks], pre[kLaneChunks];
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j) {
    const int e = lane + 64 * j;
    const bool ok = j < w.chunks && e < n_local;
    w.lo[j] = ok ? expert_offsets[e] : 0;
    w.rows[j] = ok ? expert_offsets[e + 1] - w.lo[j] : 0;
    mbs[j] = even_blocks(w.rows[j]);
  }
  const int blocks = wave_prefix(mbs, w.chunks, pre);
  const int idx = even_tile_index(blocks * n_col_blocks, vb);
  if (idx < 0) return false;
  const int base[kLaneChunks] = {0, 0, 0, 0};
  tc = wave_locate(w, mbs, base, n_col_blocks, idx, kEvenRows);
  return true;
}

}  // namespace gg
}  // namespace moe
