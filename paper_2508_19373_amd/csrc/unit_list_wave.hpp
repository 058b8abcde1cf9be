// The work list of unit_list.hpp evaluated by a wavefront instead of a scalar loop.
//
// Every workgroup of the grouped GEMM has to find its tile from expert_offsets.  The plain functions
// of unit_list.hpp walk the experts one by one, each step waiting for a scalar load: about 10 us
// per workgroup for 60 experts, a fifth of a tile's whole run time on layers with many small experts.
// Here lane l of a wavefront takes experts l, l + 64, l + 128, l + 192 (up to 256 experts), the
// running counts are wave prefix sums, and the expert that holds a given tile is found with a
// ballot.  Every result is made wave-uniform (read from one lane), and every wavefront of a
// workgroup computes the same values, so no LDS and no barrier are involved.  The functions return
// exactly what their namesakes in unit_list.hpp return; a GPU test compares the two on random
// routings through moe_debug_device_units.
#pragma once
#include "unit_list.hpp"

namespace moe {
namespace gg {

constexpr int kLaneChunks = 4;  // 256 experts / 64 lanes

// Inclusive prefix sum over the 64 lanes with data-parallel-primitive moves (a few cycles each,
// against a round trip through the LDS crossbar per step of a shuffle-based scan): shifts by 1, 2,
// 4, 8 inside each row of 16 lanes (lanes shifted in from outside the row read 0), then lane 15 of
// rows 0 and 2 is broadcast into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ inline int wave_incl_scan(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);  // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);  // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);  // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);  // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1, 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2, 3
  return v;
}

// Exclusive prefix of `len` over the experts in order (chunk j holds experts 64 j + lane); returns the total.
__device__ inline int wave_prefix(const int (&len)[kLaneChunks], int chunks, int (&pre)[kLaneChunks]) {
  int carry = 0;
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j) {
    pre[j] = 0;
    if (j < chunks) {
      const int incl = wave_incl_scan(len[j]);
      pre[j] = carry + incl - len[j];
      carry += __builtin_amdgcn_readlane(incl, 63);
    }
  }
  return carry;
}

// The expert whose interval [pre, pre + len) holds q.
struct WaveHit {
  int j, lane;
  bool found;
};
__device__ inline WaveHit wave_find(const int (&pre)[kLaneChunks], const int (&len)[kLaneChunks], int chunks, int q) {
  WaveHit h = {0, 0, false};
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j) {
    if (j < chunks && !h.found) {
      const unsigned long long m = __ballot(pre[j] <= q && q < pre[j] + len[j]);
      if (m != 0) {
        h.j = j;
        h.lane = __ffsll((long long)m) - 1;
        h.found = true;
      }
    }
  }
  return h;
}
__device__ inline int wave_pick(const int (&a)[kLaneChunks], const WaveHit& h) {
  int v = 0;
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j)
    if (j == h.j) v = __builtin_amdgcn_readlane(a[j], h.lane);
  return v;
}

// This lane's experts, and the prefix of their 256-row blocks.
struct WaveRouting {
  int chunks;
  int lo[kLaneChunks], rows[kLaneChunks];
  int n256[kLaneChunks], n128[kLaneChunks], n64[kLaneChunks];
  int pre256[kLaneChunks];
  ClassCounts cc;  // as count_tiles
};
__device__ inline WaveRouting wave_routing(const int32_t* __restrict__ expert_offsets, int n_local,
                                           int n_col_blocks, int pad_from = kPadLowTiles) {
  WaveRouting w;
  const int lane = threadIdx.x & 63;
  w.chunks = (n_local + 63) >> 6;
  int blocks = 0;  // this lane's row blocks before any padding of experts below 256 rows
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j) {
    const int e = lane + 64 * j;
    const bool ok = j < w.chunks && e < n_local;
    w.lo[j] = ok ? expert_offsets[e] : 0;
    w.rows[j] = ok ? expert_offsets[e + 1] - w.lo[j] : 0;
    blocks += row_blocks(w.rows[j], false).total();
  }
  w.cc.pad_low = __builtin_amdgcn_readlane(wave_incl_scan(blocks), 63) * n_col_blocks >= pad_from;
  int t128 = 0, t64 = 0;
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j) {
    const RowBlocks rb = row_blocks(w.rows[j], w.cc.pad_low);
    w.n256[j] = rb.n256;
    w.n128[j] = rb.n128;
    w.n64[j] = rb.n64;
    if (j < w.chunks) {
      t128 += __popcll(__ballot(rb.n128 != 0));
      t64 += __popcll(__ballot(rb.n64 != 0));
    }
  }
  const int t256 = wave_prefix(w.n256, w.chunks, w.pre256);
  w.cc.n[0] = t256 * n_col_blocks;
  w.cc.n[1] = t128 * n_col_blocks;
  w.cc.n[2] = t64 * n_col_blocks;
  return w;
}

// Tile `idx` of a list in which the lane's experts have `mbs` row blocks each, the first of them
// `base` rows into the expert: experts in order, column blocks, row blocks fastest.
__device__ inline TileCoord wave_locate(const WaveRouting& w, const int (&mbs)[kLaneChunks],
                                        const int (&base)[kLaneChunks], int n_col_blocks, int idx,
                                        int block_rows = 256) {
  int pre[kLaneChunks];
  wave_prefix(mbs, w.chunks, pre);
  const WaveHit h = wave_find(pre, mbs, w.chunks, idx / n_col_blocks);
  TileCoord t = {0, 0, 0, 0};
  if (!h.found) return t;
  const int m = wave_pick(mbs, h), lo = wave_pick(w.lo, h);
  const int local = idx - wave_pick(pre, h) * n_col_blocks;
  // (the values are uniform by construction; reading them from the first lane tells the compiler so)
  t.expert = __builtin_amdgcn_readfirstlane(h.lane + 64 * h.j);
  t.nb = __builtin_amdgcn_readfirstlane(local / m);
  t.row0 = __builtin_amdgcn_readfirstlane(lo + wave_pick(base, h) + (local % m) * block_rows);
  t.row_end = __builtin_amdgcn_readfirstlane(lo + wave_pick(w.rows, h));
  return t;
}

// locate_tile for the lists of the 128-row (cls 1) and 64-row (cls 2) remainder tiles.
__device__ inline TileCoord wave_locate_small(const WaveRouting& w, int n_col_blocks, int cls, int idx) {
  int base[kLaneChunks];
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j) base[j] = w.n256[j] * 256 + (cls == 2 ? w.n128[j] * 128 : 0);
  return cls == 1 ? wave_locate(w, w.n128, base, n_col_blocks, idx) : wave_locate(w, w.n64, base, n_col_blocks, idx);
}

// find_unit + locate_tile.  Returns false if the workgroup has no tile.
__device__ inline bool wave_find_tile(const int32_t* __restrict__ expert_offsets, int n_local, int n_col_blocks,
                                      int bid, int& cls, TileCoord& tc) {
  const WaveRouting w = wave_routing(expert_offsets, n_local, n_col_blocks);
  const Unit u = find_unit(w.cc, bid);
  if (u.cls < 0) return false;
  cls = u.cls;
  if (u.cls == 0) {
    const int base[kLaneChunks] = {0, 0, 0, 0};
    tc = wave_locate(w, w.n256, base, n_col_blocks, u.idx);
  } else {
    tc = wave_locate_small(w, n_col_blocks, u.cls, u.idx);
  }
  return true;
}

// Rows with partial sums (sliced_rows): per lane expert, the 256-row blocks that run whole and the
// number of rows behind them.
struct WaveSliced {
  int kept[kLaneChunks], cnt[kLaneChunks], pre_cnt[kLaneChunks];
  int total;
};
__device__ inline WaveSliced wave_sliced_rows(const WaveRouting& w, int keep_rb) {
  WaveSliced s;
#pragma unroll
  for (int j = 0; j < kLaneChunks; ++j) {
    s.kept[j] = min(max(keep_rb - w.pre256[j], 0), w.n256[j]);
    s.cnt[j] = w.rows[j] - min(w.rows[j], s.kept[j] * 256);
  }
  s.total = wave_prefix(s.cnt, w.chunks, s.pre_cnt);
  return s;
}

// choose_slices + find_sliced_unit + locate_full_tile / locate_tile + sliced_rows for workgroup `bid`
// of the sliced down projection.  kt0 / nk: the k-tiles of its slice; scratch_shift: for z > 0, what
// to add to a row index of the tile to get its row in the partial-sum scratch.
struct WaveSlicedUnit {
  bool valid;
  int cls, z, kt0, nk;
  TileCoord tc;
  long scratch_shift;
};
__device__ inline WaveSlicedUnit wave_find_sliced_unit(const int32_t* __restrict__ expert_offsets, int n_local,
                                                       int n_col_blocks, int nk_all, int max_slices, int bid) {
  WaveSlicedUnit r;
  r.valid = false;
  const WaveRouting w = wave_routing(expert_offsets, n_local, n_col_blocks, sliced_pad_from(nk_all));
  const SliceChoice sc = choose_slices(w.cc, n_col_blocks, nk_all, max_slices);
  const SlicedUnit u = find_sliced_unit(w.cc, sc, n_col_blocks, bid);
  if (u.cls < 0) return r;
  r.valid = true;
  r.cls = u.cls;
  r.z = u.z;
  r.kt0 = 0;
  r.nk = nk_all;
  r.scratch_shift = 0;
  if (u.cls == 1 || u.cls == 2) {
    r.tc = wave_locate_small(w, n_col_blocks, u.cls, u.idx);
  } else {
    int mbs[kLaneChunks], base[kLaneChunks];
#pragma unroll
    for (int j = 0; j < kLaneChunks; ++j) {
      const int kept = min(max(sc.keep_rb - w.pre256[j], 0), w.n256[j]);
      mbs[j] = u.cls == 3 ? kept : w.n256[j] - kept;
      base[j] = u.cls == 3 ? 0 : kept * 256;
    }
    r.tc = wave_locate(w, mbs, base, n_col_blocks, u.idx);
  }
  if (u.cls != 3) {
    r.kt0 = u.z * nk_all / sc.slices;
    r.nk = (u.z + 1) * nk_all / sc.slices - r.kt0;
    if (u.z > 0) {
      const WaveSliced s = wave_sliced_rows(w, sc.keep_rb);
      const int e = __builtin_amdgcn_readfirstlane(r.tc.expert);
      const WaveHit h = {e >> 6, e & 63, true};
      const int lo = wave_pick(w.lo, h);
      const int first = lo + min(wave_pick(w.rows, h), wave_pick(s.kept, h) * 256);
      r.scratch_shift = (long)(u.z - 1) * s.total + wave_pick(s.pre_cnt, h) - first;
    }
  }
  return r;
}

// ---- dispatch: a handful of experts are walked faster by the plain loops ---------------------------
// (the wave version costs a fixed 1-2 us of loads and cross-lane steps per workgroup, which shows on
// the short launches of expert-parallel shards with one or two experts)
constexpr int kPlainLoopExperts = 4;

__device__ inline bool find_tile(const int32_t* __restrict__ expert_offsets, int n_local, int n_col_blocks, int bid,
                                 int& cls, TileCoord& tc) {
  if (n_local > kPlainLoopExperts) return wave_find_tile(expert_offsets, n_local, n_col_blocks, bid, cls, tc);
  const ClassCounts cc = count_tiles(expert_offsets, n_local, n_col_blocks);
  const Unit u = find_unit(cc, bid);
  if (u.cls < 0) return false;
  cls = u.cls;
  tc = locate_tile(expert_offsets, n_local, n_col_blocks, u.cls, u.idx, cc.pad_low);
  return true;
}

__device__ inline WaveSlicedUnit find_sliced_unit_of(const int32_t* __restrict__ expert_offsets, int n_local,
                                                     int n_col_blocks, int nk_all, int max_slices, int bid) {
  if (n_local > kPlainLoopExperts)
    return wave_find_sliced_unit(expert_offsets, n_local, n_col_blocks, nk_all, max_slices, bid);
  WaveSlicedUnit r;
  r.valid = false;
  const ClassCounts cc = count_tiles(expert_offsets, n_local, n_col_blocks, sliced_pad_from(nk_all));
  const SliceChoice sc = choose_slices(cc, n_col_blocks, nk_all, max_slices);
  const SlicedUnit u = find_sliced_unit(cc, sc, n_col_blocks, bid);
  if (u.cls < 0) return r;
  r.valid = true;
  r.cls = u.cls;
  r.z = u.z;
  r.kt0 = 0;
  r.nk = nk_all;
  r.scratch_shift = 0;
  r.tc = (u.cls == 3 || u.cls == 0)
             ? locate_full_tile(expert_offsets, n_local, n_col_blocks, sc.keep_rb, u.cls == 0, u.idx, cc.pad_low)
             : locate_tile(expert_offsets, n_local, n_col_blocks, u.cls, u.idx, cc.pad_low);
  if (u.cls != 3) {
    r.kt0 = u.z * nk_all / sc.slices;
    r.nk = (u.z + 1) * nk_all / sc.slices - r.kt0;
    if (u.z > 0) {
      const SlicedRows sr = sliced_rows(expert_offsets, n_local, r.tc.expert, sc.keep_rb, cc.pad_low);
      r.scratch_shift = (long)(u.z - 1) * sr.total + sr.base - sr.first;
    }
  }
  return r;
}

// The rows with partial sums, for the kernel that adds them: slices (1: nothing to add), their
// number, and the row behind compact number i.
struct SumPlan {
  int slices, total, keep_rb;
  bool plain, pad_low;
  WaveRouting w;
  WaveSliced s;
};
__device__ inline SumPlan sum_plan(const int32_t* __restrict__ expert_offsets, int n_local, int n_col_blocks,
                                   int nk_all, int max_slices) {
  SumPlan p;
  p.plain = n_local <= kPlainLoopExperts;
  p.total = 0;
  p.pad_low = false;
  if (p.plain) {
    const ClassCounts cc = count_tiles(expert_offsets, n_local, n_col_blocks, sliced_pad_from(nk_all));
    const SliceChoice sc = choose_slices(cc, n_col_blocks, nk_all, max_slices);
    p.slices = sc.slices;
    p.keep_rb = sc.keep_rb;
    p.pad_low = cc.pad_low;
    if (sc.slices > 1) p.total = sliced_rows(expert_offsets, n_local, 0, sc.keep_rb, cc.pad_low).total;
  } else {
    p.w = wave_routing(expert_offsets, n_local, n_col_blocks, sliced_pad_from(nk_all));
    const SliceChoice sc = choose_slices(p.w.cc, n_col_blocks, nk_all, max_slices);
    p.slices = sc.slices;
    p.keep_rb = sc.keep_rb;
    if (sc.slices > 1) {
      p.s = wave_sliced_rows(p.w, sc.keep_rb);
      p.total = p.s.total;
    }
  }
  return p;
}
__device__ inline int sum_plan_row(const SumPlan& p, const int32_t* __restrict__ expert_offsets, int n_local, int i) {
  if (!p.plain) {
    const WaveHit h = wave_find(p.s.pre_cnt, p.s.cnt, p.w.chunks, i);
    return wave_pick(p.w.lo, h) + min(wave_pick(p.w.rows, h), wave_pick(p.s.kept, h) * 256) + i - wave_pick(p.s.pre_cnt, h);
  }
  int base = 0, before = 0;
  for (int e = 0; e < n_local; ++e) {
    const int lo = expert_offsets[e], hi = expert_offsets[e + 1];
    const int n256 = row_blocks(hi - lo, p.pad_low).n256;
    const int first = min(hi, lo + min(max(p.keep_rb - before, 0), n256) * 256);
    if (i < base + hi - first) return first + i - base;
    base += hi - first;
    before += n256;
  }
  return 0;
}

}  // namespace gg
}  // namespace moe
