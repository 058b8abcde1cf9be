// Work list of the prefill grouped GEMM: which tiles exist for a given routing, and which of
// them each workgroup runs.  Pure integer logic on expert_offsets, shared by the kernel (device)
// and by the host-side introspection call that the CPU tests use.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

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

// Work unit of one workgroup: `count` consecutive tiles of one height class, run back to back.
//
// Tiles that start together walk K in lockstep, and only then does the second reader of a weight
// panel or of an activation block find it in its XCD's L2 (the working set of 32 concurrent tiles
// leaves a k-slice resident for about two k-steps).  A short tile ends early, its compute unit
// starts the next tile out of phase, and the phase error spreads: with the remainder tiles mixed
// into the list, L2 miss traffic on ragged routing was 2.5x that of equal groups.  So units are
// made to cost about the same -- one 256-row tile, or `group` small tiles (3 x 64 rows, 2 x 128
// rows) -- and small units are spread evenly between the full ones (their weight panels come from
// HBM either way: a short tile walks K faster than its full siblings, so it never shared them).
// With `group` = 1 the small tiles run one per unit AFTER all full tiles instead: when the whole
// launch is only a few rounds deep, a fine-grained tail balances better than lockstep pays.
//
// XCD mapping: workgroup b runs on XCD b % 8 and is that XCD's slot b / 8; every XCD takes a
// contiguous eighth of the full units and an eighth of the small units.
struct Unit {
  int cls, first, count;
};
__host__ __device__ inline Unit find_unit(const ClassCounts& c, int group, int bid) {
  Unit u = {0, 0, 0};
  const int g128 = group > 1 ? 2 : 1, g64 = group;
  const int u128 = (c.n[1] + g128 - 1) / g128, u64 = (c.n[2] + g64 - 1) / g64;
  const int n_full = c.n[0], n_small = u128 + u64;
  const int c_full = (n_full + kNumXcd - 1) / kNumXcd, c_small = (n_small + kNumXcd - 1) / kNumXcd;
  const int per_xcd = c_full + c_small;
  const int xcd = bid % kNumXcd, slot = bid / kNumXcd;
  if (slot >= per_xcd) return u;
  bool is_small;
  int smalls_before;
  if (group > 1) {  // small units at the slots where floor(slot * c_small / per_xcd) steps up
    const int m0 = (int)(((long long)slot * c_small) / per_xcd);
    const int m1 = (int)(((long long)(slot + 1) * c_small) / per_xcd);
    is_small = m1 > m0;
    smalls_before = m0;
  } else {
    is_small = slot >= c_full;
    smalls_before = is_small ? slot - c_full : 0;
  }
  if (!is_small) {
    const int f = xcd * c_full + (slot - smalls_before);
    if (f < n_full) {
      u.first = f;
      u.count = 1;
    }
    return u;
  }
  int j = xcd * c_small + smalls_before;
  if (j >= n_small) return u;
  if (j < u128) {
    u.cls = 1;
    u.first = j * g128;
    u.count = c.n[1] - u.first < g128 ? c.n[1] - u.first : g128;
  } else {
    j -= u128;
    u.cls = 2;
    u.first = j * g64;
    u.count = c.n[2] - u.first < g64 ? c.n[2] - u.first : g64;
  }
  return u;
}
// Launcher's choice of `group`: remainder tiles are grouped and spread out when the launch is
// many rounds of full tiles deep on the 256 compute units, and run one per unit after the full
// tiles when it is only a few rounds.
constexpr int kComputeUnits = 256;  // MI355X
inline int small_group_for(int cap_rows, int n_col_blocks) {
  return (cap_rows / 256) * n_col_blocks >= 6 * kComputeUnits ? 3 : 1;
}
// Host-side grid size covering every unit for any routing with sum_e rows_e <= cap_rows.
inline int max_grid(int cap_rows, int n_local, int n_col_blocks) {
  const int full = (cap_rows / 256 + n_local) * n_col_blocks, small = 2 * n_local * n_col_blocks;
  return kNumXcd * ((full + kNumXcd - 1) / kNumXcd + (small + kNumXcd - 1) / kNumXcd);
}

}  // namespace gg
}  // namespace moe
