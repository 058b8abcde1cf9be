/*
 * moe_shard_debug.h -- host-only introspection of libmoe_shard, for tests.  Nothing here touches
 * the device; all pointers are HOST pointers.
 */
#ifndef MOE_SHARD_DEBUG_H
#define MOE_SHARD_DEBUG_H

#include "moe_shard.h"

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_DEBUG_UNIT_INTS 5

/*
 * The work list of moe_expert_ffn's prefill-regime grouped GEMM for one routing: the expert
 * networks run only on the rows routed to them ("MoE Model Architectures"), so the list of output
 * tiles depends on expert_offsets and is built per workgroup on the device; this call runs the
 * same code on the host.
 * expert_offsets [n_local+1] int32 HOST, non-decreasing, first >= 0, last <= cap_rows
 * n_col_blocks   column blocks per row block (GEMM1: ceil(I_s/128), GEMM2: ceil(H/256))
 * units          [max_units][MOE_DEBUG_UNIT_INTS] int32 HOST, one record per workgroup:
 *                {tile height (256/128/64, 0 = no tile), local expert, row0, row_end, column block};
 *                a tile covers rows [row0, min(row0 + height, row_end)) of its expert.
 * Returns the grid size (number of records written), or a negative MOE_ERR_* code
 * (MOE_ERR_WORKSPACE when max_units is too small).
 */
int32_t moe_debug_gemm_units(const int32_t* expert_offsets, int32_t n_local, int32_t cap_rows,
                             int32_t n_col_blocks, int32_t* units,
                             int32_t max_units);

/*
 * Which kernels moe_expert_ffn would launch for (cap_rows, shard): the paper separates a
 * memory-bound decoding regime from a compute-bound prefill regime ("Generative Inference"); the
 * library picks, per GEMM, a weight-streaming kernel or a tiled MFMA kernel from a cost estimate.
 * plan [4] int32 HOST: {GEMM1 streams weights (0/1), GEMM2 streams weights (0/1),
 *                       activation rows per streaming pass / 16 (1 or 2), K slices of GEMM2 (for a
 *                       tiled GEMM2: the most the routing can select, see moe_debug_down_slices)}
 * Returns MOE_OK or MOE_ERR_INVALID_ARG.
 */
int32_t moe_debug_ffn_plan(int32_t cap_rows, const moe_shard_t* shard, int32_t* plan);

/*
 * Row-block height of the tiled kernels moe_expert_ffn would use for (cap_rows, shard): 256 (row
 * blocks of 256 rows plus 128- and 64-row remainder tiles, moe_debug_gemm_units), or 160 (every
 * expert's rows in blocks of 160, moe_debug_even_units), which the library picks for calls with a
 * few hundred rows per expert: there a remainder tile behind one 256-row tile would stream the
 * expert's weights from HBM a second time ("Generative Inference": such launches are bound by
 * loading weights, not by compute).  Returns the height or a negative MOE_ERR_* code.
 */
int32_t moe_debug_tile_rows(int32_t cap_rows, const moe_shard_t* shard);

/*
 * The work list of the 160-row tiling, in the record format of moe_debug_gemm_units (tile height
 * 160 or 0).  Arguments and return value as there.
 */
int32_t moe_debug_even_units(const int32_t* expert_offsets, int32_t n_local, int32_t cap_rows,
                             int32_t n_col_blocks, int32_t* units, int32_t max_units);

#define MOE_DEBUG_SLICE_INTS 8

/*
 * How the tiled fp32 down projection of moe_expert_ffn is cut along K for one routing.  An
 * expert-parallel shard's load follows the routing ("Parallelism in Inference": expert parallelism
 * suffers from load imbalance), so the kernel itself decides, from expert_offsets, which tiles run
 * as several K slices on otherwise idle compute units: those of the last, partial round of 256
 * workgroups, that is the remainder tiles behind each expert's 256-row blocks and the tiles of the
 * last 256-row blocks.  This call runs the same code on the host.
 * expert_offsets [n_local+1] int32 HOST, as for moe_debug_gemm_units.
 * slices [4] int32 HOST: {256-row blocks (in expert order) whose tiles run whole, K slices of all
 *                         other tiles, rows that have partial sums, rows of partial sums
 *                         moe_ffn_workspace_bytes provides for}
 * units  NULL, or [max_units][MOE_DEBUG_SLICE_INTS] int32 HOST, one record per workgroup:
 *        {tile height (0 = no work), local expert, row0, column block, slice, first k-tile,
 *         k-tiles, scratch row its row0 is written to (-1: slice 0 writes y_perm itself)}
 * Returns the grid size, or a negative MOE_ERR_* code (MOE_ERR_WORKSPACE when max_units is too small).
 */
int32_t moe_debug_down_slices(const int32_t* expert_offsets, int32_t cap_rows, const moe_shard_t* shard,
                              int32_t* slices, int32_t* units, int32_t max_units);

#define MOE_DEBUG_DEVICE_INTS 9

/*
 * The same work lists as the two calls above, evaluated on the DEVICE by the wave-parallel code the
 * GEMM kernels use (one wavefront per workgroup id), for tests that compare it with the host code.
 * expert_offsets [n_local+1] int32 DEVICE; n_col_blocks, nk (k-tiles of 64): as the kernel is launched
 * max_slices     0: the plain list of moe_debug_gemm_units; >= 1: the sliced list of
 *                moe_debug_down_slices with that maximum; -1: the list of moe_debug_even_units
 * units          [max_units][MOE_DEBUG_DEVICE_INTS] int32 DEVICE, written asynchronously on `stream`:
 *                {tile height (0 = no work), local expert, row0, row_end, column block, slice,
 *                 first k-tile, k-tiles, scratch row of row0 (-1: writes y_perm)}
 * Returns the grid size, or a negative MOE_ERR_* code.
 */
int32_t moe_debug_device_units(const int32_t* expert_offsets, int32_t n_local, int32_t cap_rows,
                               int32_t n_col_blocks, int32_t nk, int32_t max_slices, int32_t* units,
                               int32_t max_units, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_SHARD_DEBUG_H */
