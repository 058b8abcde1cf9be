"""Host logic of moe_expert_ffn's kernel choice (CPU only, through moe_debug_ffn_plan): the
decoding regime streams weights, the prefill regime runs the tiled MFMA kernel, and launches with
too few tiles are cut along K.  The expectations below are the measured crossovers."""
import pytest

from paper_2508_19373_amd import binding as B

MIXTRAL = dict(hidden=4096, inter_full=14336, inter_slice=14336)


def _shard(E, E_loc, **kw):
    return B.make_shard(E, E_loc, 0, kw["hidden"], kw["inter_full"], kw["inter_slice"])


def test_routed_experts_switch_regime_near_twenty_rows_per_expert():
    s = _shard(8, 8, **MIXTRAL)
    # GEMM1 streams weights up to about 20 rows per expert; the down projection (K = 14336) moves to
    # the tiled kernel, cut in two along K, as soon as a pass holds 32 rows (measured 165 vs 190 us)
    for T, walk1, walk2 in ((16, True, True), (32, True, True), (64, True, False), (80, True, False),
                            (96, False, False), (128, False, False), (4096, False, False)):
        w1, w2, mt, slices = B.moe_debug_ffn_plan(T * 2, s)
        assert (w1, w2) == (walk1, walk2), T
    # up to 16 rows expected in the fullest expert: 16 rows per pass, 16 wavefronts, K = 14336 in 2 slices
    assert B.moe_debug_ffn_plan(32, s) == (True, True, 1, 2)
    assert B.moe_debug_ffn_plan(128, s)[2] == 2
    # the headline prefill shape: tiled kernels, no K slices, no scratch
    assert B.moe_debug_ffn_plan(8192, s) == (False, False, 2, 1)
    assert B.moe_ffn_workspace_bytes(8192, s) == 0


def test_single_shared_expert_never_runs_its_down_projection_on_a_handful_of_tiles():
    s = _shard(1, 1, hidden=3584, inter_full=20480, inter_slice=20480)   # H / 256 = 14 column blocks
    assert B.moe_debug_ffn_plan(32, s)[:2] == (True, True)               # decode: stream both
    for rows in (64, 128, 256, 512, 1024):
        w1, w2, mt, slices = B.moe_debug_ffn_plan(rows, s)
        assert not w1 and not w2 and slices >= 2, rows
    assert B.moe_debug_ffn_plan(256, s) == (False, False, 2, 8)
    assert B.moe_debug_ffn_plan(4096, s) == (False, False, 2, 1)          # enough tiles on their own
    assert B.moe_ffn_workspace_bytes(256, s) == 8 * 256 * 3584 * 4


def test_expert_parallel_shard_is_planned_on_its_expected_rows():
    full = _shard(8, 8, **MIXTRAL)
    ep8 = _shard(8, 1, **MIXTRAL)
    # T = 1024, k = 2: capacity 2048 rows, of which one expert of eight expects 256
    assert B.moe_debug_ffn_plan(2048, ep8)[3] == 8          # 2 row blocks x 16 column blocks: cut along K
    assert B.moe_debug_ffn_plan(2048, full)[3] == 1
    # a shard with few experts: the kernel picks the slices from the routing, and whatever it picks
    # the partial sums fit 65536 / 16 column blocks = 4096 rows
    assert B.moe_ffn_workspace_bytes(2048, ep8) == 4096 * 4096 * 4
    assert B.moe_ffn_workspace_bytes(64 * 1024, ep8) == 4096 * 4096 * 4
    assert B.moe_ffn_workspace_bytes(256, ep8) == 8 * 256 * 4096 * 4     # ... or 8 slices of the capacity
    # decode: 16 rows expected on the one local expert, but up to 128 possible: 32 rows per pass
    assert B.moe_debug_ffn_plan(128, ep8)[2] == 2
    assert B.moe_debug_ffn_plan(16, ep8)[2] == 1            # capacity itself is 16 rows


def test_down_projection_slices_follow_the_routing_on_shards_with_few_experts():
    import numpy as np
    ep4 = _shard(8, 2, **MIXTRAL)        # 16 column blocks, 224 k-tiles
    cap = 32768
    def used(*counts):
        return B.moe_debug_down_slices(np.concatenate([[0], np.cumsum(counts)]), cap, ep4)
    assert used(0, 0) == 1
    assert used(200, 100) == 8           # 2 row blocks x 16 = 32 tiles
    assert used(300, 100) == 4           # 4 row blocks (300 = 256 + 64): 64 tiles
    assert used(700, 700) == 2           # 8 row blocks (700 = 512 + 128 + 64): 128 tiles
    assert used(1100, 1000) == 1         # 10 row blocks: 160 tiles, enough on their own
    assert used(20000, 12768) == 1       # the hot shard
    # every routing that slices fits the scratch (the call returns an error otherwise)
    rng = np.random.default_rng(0)
    for _ in range(2000):
        R = int(rng.integers(0, 6000))
        a = int(rng.integers(0, R + 1))
        assert used(a, R - a) in (1, 2, 4, 8)
    # a shard with many experts, or one expert that takes every row: decided on the host
    full = _shard(8, 8, **MIXTRAL)
    assert B.moe_debug_down_slices(np.arange(9) * 10, 8192, full) == 1
    one = _shard(1, 1, hidden=3584, inter_full=20480, inter_slice=20480)
    assert B.moe_debug_down_slices([0, 10], 1024, one) == 4
    with pytest.raises(B.MoeError):
        B.moe_debug_down_slices([0, 5, 3], cap, ep4)
    with pytest.raises(B.MoeError):
        B.moe_debug_down_slices([0, 5, cap + 1], cap, ep4)


def test_k_extents_without_a_fast_streaming_kernel_go_to_the_tiled_kernel_early():
    # Qwen1.5-MoE under TP 4: the padded slice is 384 wide, a K extent only the generic streaming kernel covers
    s = B.make_shard(60, 60, 0, 2048, 1536, 384)
    w1, w2, mt, slices = B.moe_debug_ffn_plan(64 * 4, s)
    assert w1 and not w2


def test_invalid_arguments():
    L = B.lib()
    import ctypes
    plan = (ctypes.c_int32 * 4)()
    s = _shard(8, 8, **MIXTRAL)
    assert L.moe_debug_ffn_plan(-1, ctypes.byref(s), plan) == B.MOE_ERR_INVALID_ARG
    assert L.moe_debug_ffn_plan(8, None, plan) == B.MOE_ERR_INVALID_ARG
    assert L.moe_debug_ffn_plan(8, ctypes.byref(s), None) == B.MOE_ERR_INVALID_ARG
