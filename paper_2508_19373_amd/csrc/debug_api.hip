// Host-only introspection of the prefill grouped GEMM's work list (no device work): runs the same
// integer logic the kernel runs per workgroup, so CPU tests can check that every tile of every
// routing is covered exactly once.
#include "moe_shard_debug.h"
#include "moe_internal.hpp"
#include "unit_list_even.hpp"
#include "unit_list_wave.hpp"

extern "C" int32_t moe_debug_gemm_units(const int32_t* expert_offsets, int32_t n_local, int32_t cap_rows,
                                        int32_t n_col_blocks, int32_t* units,
                                        int32_t max_units) {
  using namespace moe::gg;
  if (expert_offsets == nullptr || units == nullptr || n_local < 1 || cap_rows < 0 || n_col_blocks < 1)
    return MOE_ERR_INVALID_ARG;
  for (int e = 0; e < n_local; ++e)
    if (expert_offsets[e] > expert_offsets[e + 1]) return MOE_ERR_INVALID_ARG;
  if (expert_offsets[0] < 0 || expert_offsets[n_local] > cap_rows) return MOE_ERR_INVALID_ARG;
  const int grid = max_grid(cap_rows, n_local, n_col_blocks);
  if (grid > max_units) return MOE_ERR_WORKSPACE;
  const ClassCounts cc = count_tiles(expert_offsets, n_local, n_col_blocks);
  for (int b = 0; b < grid; ++b) {
    int32_t* rec = units + (size_t)b * MOE_DEBUG_UNIT_INTS;
    for (int i = 0; i < MOE_DEBUG_UNIT_INTS; ++i) rec[i] = 0;
    const Unit u = find_unit(cc, b);
    if (u.cls < 0) continue;
    const TileCoord tc = locate_tile(expert_offsets, n_local, n_col_blocks, u.cls, u.idx, cc.pad_low);
    rec[0] = u.cls == 0 ? 256 : (u.cls == 1 ? 128 : 64);
    rec[1] = tc.expert;
    rec[2] = tc.row0;
    rec[3] = tc.row_end;
    rec[4] = tc.nb;
  }
  return grid;
}

extern "C" int32_t moe_debug_ffn_plan(int32_t cap_rows, const moe_shard_t* shard, int32_t* plan) {
  if (cap_rows < 0 || shard == nullptr || plan == nullptr) return MOE_ERR_INVALID_ARG;
  if (shard->n_experts < 1 || shard->n_local_experts < 1 || shard->n_local_experts > shard->n_experts ||
      shard->hidden < 64 || shard->inter_slice < 64)
    return MOE_ERR_INVALID_ARG;
  moe::ffn_plan(cap_rows, moe::expected_rows(cap_rows, shard), shard->n_local_experts, shard->hidden,
                shard->inter_slice, plan);
  return MOE_OK;
}

extern "C" int32_t moe_debug_tile_rows(int32_t cap_rows, const moe_shard_t* shard) {
  if (cap_rows < 0 || shard == nullptr) return MOE_ERR_INVALID_ARG;
  if (shard->n_experts < 1 || shard->n_local_experts < 1 || shard->n_local_experts > shard->n_experts ||
      shard->hidden < 64 || shard->inter_slice < 64)
    return MOE_ERR_INVALID_ARG;
  return moe::tiled_block_rows(cap_rows, moe::expected_rows(cap_rows, shard), shard->n_local_experts, shard->hidden,
                               shard->inter_slice);
}

extern "C" int32_t moe_debug_even_units(const int32_t* expert_offsets, int32_t n_local, int32_t cap_rows,
                                        int32_t n_col_blocks, int32_t* units, int32_t max_units) {
  using namespace moe::gg;
  if (expert_offsets == nullptr || units == nullptr || n_local < 1 || cap_rows < 0 || n_col_blocks < 1)
    return MOE_ERR_INVALID_ARG;
  for (int e = 0; e < n_local; ++e)
    if (expert_offsets[e] > expert_offsets[e + 1]) return MOE_ERR_INVALID_ARG;
  if (expert_offsets[0] < 0 || expert_offsets[n_local] > cap_rows) return MOE_ERR_INVALID_ARG;
  const int grid = even_max_ids(cap_rows, n_local, n_col_blocks);
  if (grid > max_units) return MOE_ERR_WORKSPACE;
  const int n_tiles = even_tiles(expert_offsets, n_local, n_col_blocks);
  for (int b = 0; b < grid; ++b) {
    int32_t* rec = units + (size_t)b * MOE_DEBUG_UNIT_INTS;
    for (int i = 0; i < MOE_DEBUG_UNIT_INTS; ++i) rec[i] = 0;
    const int idx = even_tile_index(n_tiles, b);
    if (idx < 0) continue;
    const TileCoord tc = even_locate(expert_offsets, n_local, n_col_blocks, idx);
    rec[0] = kEvenRows;
    rec[1] = tc.expert;
    rec[2] = tc.row0;
    rec[3] = tc.row_end;
    rec[4] = tc.nb;
  }
  return grid;
}

extern "C" int32_t moe_debug_down_slices(const int32_t* expert_offsets, int32_t cap_rows, const moe_shard_t* shard,
                                         int32_t* slices, int32_t* units, int32_t max_units) {
  if (expert_offsets == nullptr || cap_rows < 0 || shard == nullptr || slices == nullptr) return MOE_ERR_INVALID_ARG;
  if (shard->n_experts < 1 || shard->n_local_experts < 1 || shard->n_local_experts > shard->n_experts ||
      shard->hidden < 64 || shard->inter_slice < 64)
    return MOE_ERR_INVALID_ARG;
  const int n_local = shard->n_local_experts;
  for (int e = 0; e < n_local; ++e)
    if (expert_offsets[e] > expert_offsets[e + 1]) return MOE_ERR_INVALID_ARG;
  if (expert_offsets[0] < 0 || expert_offsets[n_local] > cap_rows) return MOE_ERR_INVALID_ARG;
  using namespace moe::gg;
  const int ncb = (shard->hidden + 255) / 256, nk = shard->inter_slice / 64;
  const SlicePlan sp = slice_plan(cap_rows, ncb, shard->inter_slice);
  const ClassCounts cc = count_tiles(expert_offsets, n_local, ncb, sp.max_slices > 1 ? sliced_pad_from(nk) : kPadLowTiles);
  const SliceChoice sc = choose_slices(cc, ncb, nk, sp.max_slices);
  slices[0] = sc.keep_rb;
  slices[1] = sc.slices;
  slices[2] = sc.slices > 1 ? sliced_rows(expert_offsets, n_local, 0, sc.keep_rb, cc.pad_low).total : 0;
  slices[3] = sp.scratch_rows;
  const int grid = sp.max_slices > 1 ? sliced_grid(cap_rows, n_local, ncb) : max_grid(cap_rows, n_local, ncb);
  if (units == nullptr) return grid;
  if (grid > max_units) return MOE_ERR_WORKSPACE;
  for (int b = 0; b < grid; ++b) {
    int32_t* rec = units + (size_t)b * MOE_DEBUG_SLICE_INTS;
    for (int i = 0; i < MOE_DEBUG_SLICE_INTS; ++i) rec[i] = 0;
    const SlicedUnit u = find_sliced_unit(cc, sc, ncb, b);
    if (u.cls < 0) continue;
    const TileCoord tc = (u.cls == 3 || u.cls == 0)
                             ? locate_full_tile(expert_offsets, n_local, ncb, sc.keep_rb, u.cls == 0, u.idx, cc.pad_low)
                             : locate_tile(expert_offsets, n_local, ncb, u.cls, u.idx, cc.pad_low);
    const int s = u.cls == 3 ? 1 : sc.slices;
    const int kt0 = u.z * nk / s;
    const SlicedRows sr = sliced_rows(expert_offsets, n_local, tc.expert, sc.keep_rb, cc.pad_low);
    rec[0] = (u.cls == 3 || u.cls == 0) ? 256 : (u.cls == 1 ? 128 : 64);
    rec[1] = tc.expert;
    rec[2] = tc.row0;
    rec[3] = tc.nb;
    rec[4] = u.z;
    rec[5] = kt0;
    rec[6] = (u.z + 1) * nk / s - kt0;
    rec[7] = u.z == 0 ? -1 : (u.z - 1) * sr.total + sr.base + tc.row0 - sr.first;
  }
  return grid;
}

namespace {
// One wavefront per workgroup id of the GEMM grid: the record the GEMM kernels would act on.
__global__ __launch_bounds__(64) void device_units_kernel(const int32_t* __restrict__ expert_offsets, int n_local,
                                                         int n_col_blocks, int nk, int max_slices,
                                                         int32_t* __restrict__ units) {
  using namespace moe::gg;
  int32_t rec[MOE_DEBUG_DEVICE_INTS] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
  if (max_slices < 0) {
    TileCoord tc;
    if (even_find_tile(expert_offsets, n_local, n_col_blocks, blockIdx.x, tc)) {
      rec[0] = kEvenRows;
      rec[1] = tc.expert;
      rec[2] = tc.row0;
      rec[3] = tc.row_end;
      rec[4] = tc.nb;
      rec[7] = nk;
      rec[8] = -1;
    }
  } else if (max_slices == 0) {
    int cls = 0;
    TileCoord tc;
    if (find_tile(expert_offsets, n_local, n_col_blocks, blockIdx.x, cls, tc)) {
      rec[0] = cls == 0 ? 256 : (cls == 1 ? 128 : 64);
      rec[1] = tc.expert;
      rec[2] = tc.row0;
      rec[3] = tc.row_end;
      rec[4] = tc.nb;
      rec[7] = nk;
      rec[8] = -1;
    }
  } else {
    const WaveSlicedUnit u = find_sliced_unit_of(expert_offsets, n_local, n_col_blocks, nk, max_slices, blockIdx.x);
    if (u.valid) {
      rec[0] = (u.cls == 3 || u.cls == 0) ? 256 : (u.cls == 1 ? 128 : 64);
      rec[1] = u.tc.expert;
      rec[2] = u.tc.row0;
      rec[3] = u.tc.row_end;
      rec[4] = u.tc.nb;
      rec[5] = u.z;
      rec[6] = u.kt0;
      rec[7] = u.nk;
      rec[8] = u.z == 0 ? -1 : (int32_t)(u.scratch_shift + u.tc.row0);
    }
  }
  if (threadIdx.x == 0)
    for (int i = 0; i < MOE_DEBUG_DEVICE_INTS; ++i) units[(size_t)blockIdx.x * MOE_DEBUG_DEVICE_INTS + i] = rec[i];
}
}  // namespace

extern "C" int32_t moe_debug_device_units(const int32_t* expert_offsets, int32_t n_local, int32_t cap_rows,
                                          int32_t n_col_blocks, int32_t nk, int32_t max_slices, int32_t* units,
                                          int32_t max_units, void* stream) {
  using namespace moe::gg;
  if (expert_offsets == nullptr || units == nullptr || n_local < 1 || n_local > MOE_MAX_EXPERTS || cap_rows < 0 ||
      n_col_blocks < 1 || nk < 1 || max_slices < -1 || max_slices > 16)
    return MOE_ERR_INVALID_ARG;
  const int grid = max_slices < 0 ? even_max_ids(cap_rows, n_local, n_col_blocks)
                                  : (max_slices > 0 ? sliced_grid(cap_rows, n_local, n_col_blocks)
                                                    : max_grid(cap_rows, n_local, n_col_blocks));
  if (grid > max_units) return MOE_ERR_WORKSPACE;
  hipLaunchKernelGGL(device_units_kernel, dim3(grid), dim3(64), 0, static_cast<hipStream_t>(stream), expert_offsets,
                     n_local, n_col_blocks, nk, max_slices, units);
  return hipGetLastError() == hipSuccess ? grid : MOE_ERR_HIP;
}
