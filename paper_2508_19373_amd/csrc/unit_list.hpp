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

// Row blocks of one expert: as many 256-row blocks as fit; a remainder of up to 64 rows is one
// 64-row block, of up to 128 rows one 128-row block.  A larger remainder is padded to one more
// 256-row block if the expert has a 256-row block already: a remainder tile re-streams the expert's
// weights from HBM, which costs about as much chip time as the MFMA work of a 256-row block that
// shares them in L2 with its siblings, and 128 + 64 rows would stream them twice.  An expert with
// 129 to 192 rows has no sibling to share with.  In a launch that fills the chip (`pad_low`, see
// count_tiles) it is padded to one 256-row block all the same, because that launch is bound by HBM
// and the second stream is pure loss (Mixtral at 128 rows per expert: 892 -> 673 us per layer); in
// a launch short of tiles it keeps 128 + 64, whose deeper pipelines stream faster per compute unit
// (a single expert of 181 rows: GEMM1 72 against 81 us).
struct RowBlocks {
  int n256, n128, n64;
  __host__ __device__ inline int total() const { return n256 + n128 + n64; }
};
__host__ __device__ inline RowBlocks row_blocks(int rows, bool pad_low) {
  RowBlocks rb;
  const int q = rows >> 8, r = rows & 255;
  const int pad = (q > 0 || pad_low) ? 128 : 192;  // remainders above this become a 256-row block
  rb.n256 = q + (r > pad ? 1 : 0);
  rb.n128 = (r > 64 && r <= pad) ? 1 : 0;
  rb.n64 = ((r > 0 && r <= 64) || (r > 128 && r <= pad)) ? 1 : 0;
  return rb;
}

struct TileCoord {
  int expert, row0, row_end, nb;
};

// Tiles per height class (0: 256 rows, 1: 128, 2: 64), over all local experts and column blocks.
// pad_low: the launch has at least 256 tiles before any padding of experts below 256 rows, that is,
// it fills every compute unit (every function below takes the flag from here).
struct ClassCounts {
  int n[3];
  bool pad_low;
};
constexpr int kPadLowTiles = 256;
// The sliced down projection pads from 128 tiles on (sliced_pad_from): its tiles are cut along K until they fill the
// chip anyway, so 128 + 64 rows only stream an expert's weights twice (Mixtral at 128 to 200 rows
// per expert: 224 tiles, below kPadLowTiles; down projection 262 / 311 us at 512 / 768 tokens
// against 171 us at 384).  With fewer tiles the padded launch needs so many slices per tile to
// fill the chip that the walks are mostly fixed cost (192 rows per expert: one expert, 32 tiles,
// layer 150 -> 157 us when padded; two experts, 64 tiles, 225 -> 228 us; four, 128 tiles, 430 -> 393 us).
// Nor does it pay on a short K (below 48 k-tiles): there is little to re-stream, and the two slices
// that 128 padded tiles allow are short (Mixtral TP=8, 28 k-tiles: layer 151 -> 162 us at 512 tokens,
// 179 -> 172 us at 768).
__host__ __device__ inline int sliced_pad_from(int nk) { return nk >= 48 ? 128 : kPadLowTiles; }
__host__ __device__ inline ClassCounts count_tiles(const int32_t* __restrict__ expert_offsets, int n_local,
                                                   int n_col_blocks, int pad_from = kPadLowTiles) {
  ClassCounts c = {{0, 0, 0}, false};
  int blocks = 0;
  for (int e = 0; e < n_local; ++e) blocks += row_blocks(expert_offsets[e + 1] - expert_offsets[e], false).total();
  c.pad_low = blocks * n_col_blocks >= pad_from;
  for (int e = 0; e < n_local; ++e) {
    const RowBlocks rb = row_blocks(expert_offsets[e + 1] - expert_offsets[e], c.pad_low);
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
                                                 int n_col_blocks, int cls, int idx, bool pad_low) {
  TileCoord t = {0, 0, 0, 0};
  for (int e = 0; e < n_local; ++e) {
    const int lo = expert_offsets[e], hi = expert_offsets[e + 1];
    const RowBlocks rb = row_blocks(hi - lo, pad_low);
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
// final round; they run last expert first, because what the full tiles streamed most recently is what
// the 256 MB memory-side cache still holds (Qwen1.5 at 4096 tokens -1.5 % on two boxes; Mixtral,
// where one expert's weights fill that cache, -0.1 to -0.8 %).  Spreading remainder tiles between the full ones in groups that cost about one
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
        // remainder tiles run last expert first: what the full tiles streamed most recently is
        // what the memory-side cache still holds
        u.idx = cls == 0 ? idx : c.n[cls] - 1 - idx;
      }
      return u;
    }
    slot -= chunk;
  }
  return u;
}
// ---- K slices of the fp32 down projection, decided from the routing -------------------------------
// One workgroup per tile leaves compute units idle for a whole walk over K whenever the tiles do
// not fill a round of 256: a launch with few tiles (a single shared expert, the cold shard of a
// skewed expert-parallel split), the last round of the 256-row tiles (544 tiles are 2.1 rounds and
// take 3), and the remainder phase, where the last rows of every expert are 128- or 64-row tiles
// that re-stream the expert's weights latency-bound.  The tiles of that last round are
// therefore cut along K into slices that run as separate workgroups: the remainder tiles and the
// 256-row tiles of the last row blocks (in expert order), as many whole row blocks as the last
// round holds.  Slice 0 writes y, slice z >= 1 writes fp32 partial sums that a second kernel adds
// to y in slice order.
//
// fit_slices: the number of slices s <= min(max_slices, 256 / n_tiles, nk / 8) that minimises an
// estimate of the run time, in sixteenths of one k-tile step (1.1-1.3 us): the walk, nk / s, and
// for s > 1 the second kernel, 4 steps for its launch plus rows * n_col_blocks * (s + 1) / 4400 for
// reading s - 1 partial sums of `rows` rows and updating y at about 4 TB/s.  (Measured: 120
// remainder tiles of 22 k-tiles and 1500 rows are not worth cutting in two, 16 tiles of 88 k-tiles
// and 512 rows are worth cutting in 11.)
__host__ __device__ inline int fit_slices(int n_tiles, int nk, int max_slices, int rows, int n_col_blocks) {
  if (n_tiles <= 0) return 1;
  int hi = 256 / n_tiles;
  if (hi > max_slices) hi = max_slices;
  if (hi > nk / 8) hi = nk / 8;
  int best = 1, best_cost = nk * 16;
  for (int s = 2; s <= hi; ++s) {
    const int cost = (nk * 16 + s - 1) / s + 64 + rows * n_col_blocks * (s + 1) / 275;
    if (cost < best_cost) best = s, best_cost = cost;
  }
  return best;
}
// keep_rb: 256-row blocks (counted over the experts in order) whose tiles run whole; the tiles of
// all later 256-row blocks and all remainder tiles run in `slices` K slices.
struct SliceChoice {
  int keep_rb, slices;
};
__host__ __device__ inline SliceChoice choose_slices(const ClassCounts& c, int n_col_blocks, int nk,
                                                     int max_slices) {
  const int n_rb = c.n[0] / n_col_blocks, n_small = c.n[1] + c.n[2];
  const int small_rows = c.n[1] / n_col_blocks * 128 + c.n[2] / n_col_blocks * 64;  // at most
  int tail_rb = 0;
  if (c.n[0] + n_small <= 128) {
    tail_rb = n_rb;  // less than half a round in all
  } else {
    const int last = c.n[0] % 256;  // 256-row tiles in the last, partial round
    if (last > 0 && last <= 128) tail_rb = (last + n_col_blocks - 1) / n_col_blocks;
  }
  SliceChoice sc;
  sc.slices = fit_slices(tail_rb * n_col_blocks + n_small, nk, max_slices, tail_rb * 256 + small_rows, n_col_blocks);
  if (sc.slices == 1 && n_small > 0 && tail_rb > 0) {
    sc.slices = fit_slices(n_small, nk, max_slices, small_rows, n_col_blocks);
    tail_rb = 0;
  }
  sc.keep_rb = sc.slices > 1 ? n_rb - tail_rb : n_rb;
  return sc;
}
constexpr int kMaxKSlices = 16;
inline int max_k_slices(int K) {
  const int s = K / 64 / 8;
  return s > kMaxKSlices ? kMaxKSlices : (s < 1 ? 1 : s);
}
// Workgroup -> (tile, slice).  Order: the whole 256-row tiles as in find_unit; then the sliced
// 256-row tiles, the 128-row and the 64-row tiles, each list repeated once per slice, all tiles of
// slice 0 first (tiles of one slice walk the same k range, so they share weight panels).
struct SlicedUnit {
  int cls, idx, z;  // cls: 0/1/2 height class, 3 = whole 256-row tile (z = 0)
};
__host__ __device__ inline SlicedUnit find_sliced_unit(const ClassCounts& c, const SliceChoice& sc, int n_col_blocks,
                                                       int bid) {
  const int kept = sc.keep_rb * n_col_blocks;
  const int n[4] = {kept, c.n[0] - kept, c.n[1], c.n[2]};
  SlicedUnit r = {-1, 0, 0};
  const int xcd = bid % kNumXcd;
  int slot = bid / kNumXcd;
  for (int v = 0; v < 4; ++v) {
    const int m = v == 0 ? n[0] : n[v] * sc.slices;
    const int chunk = (m + kNumXcd - 1) / kNumXcd;
    if (slot < chunk) {
      const int i = xcd * chunk + slot;
      if (i < m) {
        r.cls = v == 0 ? 3 : v - 1;
        r.z = i / n[v];
        r.idx = v < 2 ? i % n[v] : n[v] - 1 - i % n[v];  // remainder tiles: last expert first, as in find_unit
      }
      return r;
    }
    slot -= chunk;
  }
  return r;
}
// 256-row tile `idx` among the whole ones (tail = false) or among the sliced ones (tail = true):
// experts in order, column blocks, row blocks fastest, as locate_tile.
__host__ __device__ inline TileCoord locate_full_tile(const int32_t* __restrict__ expert_offsets, int n_local,
                                                      int n_col_blocks, int keep_rb, bool tail, int idx,
                                                      bool pad_low) {
  TileCoord t = {0, 0, 0, 0};
  int before = 0;
  for (int e = 0; e < n_local; ++e) {
    const int lo = expert_offsets[e], hi = expert_offsets[e + 1];
    const int n256 = row_blocks(hi - lo, pad_low).n256;
    const int kept = min(max(keep_rb - before, 0), n256);
    const int mbs = tail ? n256 - kept : kept;
    const int tiles = mbs * n_col_blocks;
    if (idx < tiles) {
      t.expert = e;
      t.nb = idx / mbs;
      t.row_end = hi;
      t.row0 = lo + (idx % mbs + (tail ? kept : 0)) * 256;
      return t;
    }
    idx -= tiles;
    before += n256;
  }
  return t;
}
// Rows that have partial sums, numbered compactly over the experts: each expert's rows behind its
// whole 256-row blocks.  For expert e: `first` is its first such row and `base` that row's compact
// number; `total` counts them over the shard.  Slice z >= 1 keeps the partial sums of compact row i
// at row (z - 1) * total + i of the scratch: (slices - 1) * total <= 65536 / n_col_blocks rows,
// since slices * tiles <= 256 and a tile has at most 256 rows.
struct SlicedRows {
  int base, first, total;
};
__host__ __device__ inline SlicedRows sliced_rows(const int32_t* __restrict__ expert_offsets, int n_local, int e,
                                                  int keep_rb, bool pad_low) {
  SlicedRows r = {0, 0, 0};
  int before = 0;
  for (int i = 0; i < n_local; ++i) {
    const int lo = expert_offsets[i], hi = expert_offsets[i + 1];
    const int n256 = row_blocks(hi - lo, pad_low).n256;
    const int first = min(hi, lo + min(max(keep_rb - before, 0), n256) * 256);
    if (i == e) {
      r.base = r.total;
      r.first = first;
    }
    r.total += hi - first;
    before += n256;
  }
  return r;
}
inline int sliced_scratch_rows(int cap_rows, int n_col_blocks, int max_slices) {
  const long a = 65536 / n_col_blocks, b = (long)(max_slices - 1) * cap_rows;
  return (int)(a < b ? a : b);
}
// Host-side grid size covering every tile for any routing with sum_e rows_e <= cap_rows: at most
// cap_rows/256 + n_local full row blocks, and one 128-row and one 64-row block per expert.
inline int max_grid(int cap_rows, int n_local, int n_col_blocks) {
  const int full = (cap_rows / 256 + n_local) * n_col_blocks, small = n_local * n_col_blocks;
  return kNumXcd * ((full + kNumXcd - 1) / kNumXcd + 2 * ((small + kNumXcd - 1) / kNumXcd));
}

// Grid of the sliced kernel: the whole tiles, then three lists that either are cut along K (then
// they have at most 256 workgroups together, 35 per XCD with the rounding of each list) or are the
// plain 128- and 64-row lists.
inline int sliced_grid(int cap_rows, int n_local, int n_col_blocks) {
  const int full = (cap_rows / 256 + n_local) * n_col_blocks, small = n_local * n_col_blocks;
  int rest = 2 * ((small + kNumXcd - 1) / kNumXcd);
  if (rest < 256 / kNumXcd + 3) rest = 256 / kNumXcd + 3;
  return kNumXcd * ((full + kNumXcd - 1) / kNumXcd + rest);
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

// How a tiled fp32 down projection may be cut along K: up to `max_slices` (1: never), chosen per
// routing on the device (choose_slices); scratch_rows: rows of fp32 partial sums it needs room for.
struct SlicePlan {
  int max_slices, scratch_rows;
};
inline SlicePlan slice_plan(int cap_rows, int n_col_blocks, int K) {
  const int s = max_k_slices(K);
  return SlicePlan{s, s > 1 ? sliced_scratch_rows(cap_rows, n_col_blocks, s) : 0};
}

}  // namespace gg
}  // namespace moe
