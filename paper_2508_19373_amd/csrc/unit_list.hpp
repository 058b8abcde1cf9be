// Work list of the prefill grouped GEMM: which tiles exist for a given routing, and which of
// them each workgroup runs.  Pure integer logic on expert_offsets, shared by the kernel (device)
// and by the host-side introspection call that the CPU tests use.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>

namespace moe {
namespace gg {

constexpr int kNumXcd = 8;

// Row blocks of one expert: as many 256-row blocks as fit, then the remainder r is covered by
// the cheapest of {64}, {128}, {128 + 64}, {256} rows, so the padding per expert is below 64
// rows (padded rows are pure loss: only algorithmic FLOPs count).
struct RowBlocks {
  int n256, n128, n64;
  __host__ __device__ inline int total() const { return n256 + n128 + n64; }
};
__host__ __device__ inline RowBlocks row_blocks(int rows) {
  RowBlocks rb;
  const int r = rows & 255;
  rb.n256 = (rows >> 8) + (r > 192 ? 1 : 0);
  rb.n128 = (r > 64 && r <= 192) ? 1 : 0;
  rb.n64 = ((r > 0 && r <= 64) || (r > 128 && r <= 192)) ? 1 : 0;
  return rb;
}

struct TileCoord {
  int expert, row0, row_end, nb;
};

// Tiles per height class (0: 256 rows, 1: 128, 2: 64), over all local experts and column blocks.
struct ClassCounts {
  int n[3];
};
__host__ __device__ inline ClassCounts count_tiles(const int32_t* __restrict__ expert_offsets, int n_local,
                                                   int n_col_blocks) {
  ClassCounts c = {{0, 0, 0}};
  for (int e = 0; e < n_local; ++e) {
    const RowBlocks rb = row_blocks(expert_offsets[e + 1] - expert_offsets[e]);
    c.n[0] += rb.n256 * n_col_blocks;
    c.n[1] += rb.n128 * n_col_blocks;
    c.n[2] += rb.n64 * n_col_blocks;
  }
  return c;
}

// Tile `idx` of height class `cls`: experts in order, inside an expert column blocks in order,
// inside a column block the row blocks of that class (row block fastest, so neighbours share the
// weight panel and a run of tiles covers all full row blocks of a few column blocks).
__host__ __device__ inline TileCoord locate_tile(const int32_t* __restrict__ expert_offsets, int n_local,
                                                 int n_col_blocks, int cls, int idx) {
  TileCoord t = {0, 0, 0, 0};
  for (int e = 0; e < n_local; ++e) {
    const int lo = expert_offsets[e], hi = expert_offsets[e + 1];
    const RowBlocks rb = row_blocks(hi - lo);
    const int mbs = cls == 0 ? rb.n256 : (cls == 1 ? rb.n128 : rb.n64);
    const int tiles = mbs * n_col_blocks;
    if (idx < tiles) {
      t.expert = e;
      t.nb = idx / mbs;
      t.row_end = hi;
      t.row0 = lo + (cls == 0 ? (idx % mbs) * 256 : (cls == 1 ? rb.n256 * 256 : rb.n256 * 256 + rb.n128 * 128));
      return t;
    }
    idx -= tiles;
  }
  return t;
}

// Tile of workgroup `bid`, or cls < 0 if it has none.
//
// Order: all 256-row tiles first, then the 128-row, then the 64-row remainder tiles.  Tiles that
// start together walk K in lockstep, and only then does the second reader of a weight panel or an
// activation block find it in its XCD's L2 (the working set of 32 concurrent tiles leaves a
// k-slice resident for about two k-steps).  A short tile ends early, its compute unit starts the
// next tile out of phase, and the phase error spreads: with remainder tiles mixed into the list,
// L2 miss traffic on ragged routing was 2.5x that of equal groups (and a short tile walks K
// faster than its full siblings, so it never shared their weight panel anyway).  With the short
// tiles last, the full tiles run as they do for equal groups, and the small tiles balance the
// final round.  Spreading remainder tiles between the full ones in groups that cost about one
// full tile measured worse (traffic 6.2 GB against 4.0 GB, 2 % slower).
//
// XCD mapping: workgroup b runs on XCD b % 8 and is that XCD's slot b / 8; every XCD takes a
// contiguous eighth of each class, largest tiles first.
struct Unit {
  int cls, idx;
};
__host__ __device__ inline Unit find_unit(const ClassCounts& c, int bid) {
  Unit u = {-1, 0};
  const int xcd = bid % kNumXcd;
  int slot = bid / kNumXcd;
  for (int cls = 0; cls < 3; ++cls) {
    const int chunk = (c.n[cls] + kNumXcd - 1) / kNumXcd;
    if (slot < chunk) {
      const int idx = xcd * chunk + slot;
      if (idx < c.n[cls]) {
        u.cls = cls;
        u.idx = idx;
      }
      return u;
    }
    slot -= chunk;
  }
  return u;
}
// K slices a down projection with `n_tiles` tiles of `nk` k-tiles uses out of the `max_slices` (a
// power of two) that were launched: as many as keep the launch within 256 workgroups with at least 8
// k-tiles each.  Decided on the device from the actual routing, so that a shard that received far
// fewer rows than its share still fills the chip (the cold shard of a skewed expert-parallel
// split).  The partial sums of slice z start at row z * R of the scratch buffer, R the shard's
// actual rows: slices * R <= slices * n_tiles * 256 / n_col_blocks <= 65536 / n_col_blocks rows.
__host__ __device__ inline int adaptive_slices(int n_tiles, int nk, int max_slices) {
  if (n_tiles <= 0) return 1;
  for (int s = max_slices; s >= 2; s >>= 1)
    if (n_tiles * s <= 256 && nk % s == 0 && nk / s >= 8) return s;
  return 1;
}
// Shards with few experts and few column blocks can end up with few tiles whatever their capacity:
// for them the slicing is adaptive.
inline bool adaptive_slicing(int n_local, int n_col_blocks) { return n_local * n_col_blocks <= 64; }
inline int max_k_slices(int K) {
  const int nk = K / 64;
  for (int s = 8; s >= 2; s >>= 1)
    if (nk % s == 0 && nk / s >= 8) return s;
  return 1;
}
inline int adaptive_scratch_rows(int cap_rows, int n_col_blocks, int max_slices) {
  const long a = 65536 / n_col_blocks, b = (long)max_slices * cap_rows;
  return (int)(a < b ? a : b);
}
// Host-side grid size covering every tile for any routing with sum_e rows_e <= cap_rows: at most
// cap_rows/256 + n_local full row blocks, and one 128-row and one 64-row block per expert.
inline int max_grid(int cap_rows, int n_local, int n_col_blocks) {
  const int full = (cap_rows / 256 + n_local) * n_col_blocks, small = n_local * n_col_blocks;
  return kNumXcd * ((full + kNumXcd - 1) / kNumXcd + 2 * ((small + kNumXcd - 1) / kNumXcd));
}

// Tiles a launch is expected to have: every local expert with its expected rows plus a two-sigma
// margin (none when `exact`: one expert that takes every row), in 256-row blocks (a remainder tile
// counts as a block).
inline int expected_tiles(int est_rows, int n_local, int n_col_blocks, bool exact) {
  const double avg = (double)est_rows / n_local;
  const int blocks = (int)((avg + (exact ? 0.0 : 2.0 * sqrt(avg)) + 255.0) / 256.0);
  return n_local * (blocks < 1 ? 1 : blocks) * n_col_blocks;
}

// K slices for a down projection whose tile count would leave most compute units idle (a single
// shared expert with a few hundred rows: H / 256 column blocks per row block): the largest of 8, 4,
// 2 that divides the k-tile count, keeps at least 8 k-tiles per slice and at most 256 workgroups.
inline int k_slices_for(int est_rows, int n_local, int n_col_blocks, int K, bool exact) {
  const int tiles = expected_tiles(est_rows, n_local, n_col_blocks, exact), nk = K / 64;
  for (int s = 8; s >= 2; s >>= 1)
    if (tiles * s <= 256 && nk % s == 0 && nk / s >= 8) return s;
  return 1;
}

// How a tiled down projection is cut along K: `slices` are launched (1: unsliced); if `adaptive`
// the kernel decides from the routing how many of them it uses (adaptive_slices), else all are used.
// scratch_rows: rows of fp32 partial sums the launch needs room for.
struct SlicePlan {
  int slices;
  bool adaptive;
  int scratch_rows;
};
inline SlicePlan slice_plan(int cap_rows, int est_rows, int n_local, int n_col_blocks, int K) {
  const bool exact = n_local == 1 && est_rows == cap_rows;  // one expert that takes every row
  if (!exact && adaptive_slicing(n_local, n_col_blocks)) {
    const int s = max_k_slices(K);
    return SlicePlan{s, s > 1, s > 1 ? adaptive_scratch_rows(cap_rows, n_col_blocks, s) : 0};
  }
  const int s = k_slices_for(est_rows, n_local, n_col_blocks, K, exact);
  return SlicePlan{s, false, s > 1 ? s * cap_rows : 0};
}

}  // namespace gg
}  // namespace moe
