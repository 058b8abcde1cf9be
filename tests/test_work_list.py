"""Host logic of the prefill grouped GEMM: the per-workgroup tile list, run on the CPU through
moe_debug_gemm_units.  For any routing, the tiles of all workgroups must cover every routed row of
every column block exactly once, never reach into another expert's rows, and the grid bound the
launcher uses must hold."""
import ctypes

import numpy as np

from paper_2508_19373_amd import binding as B


def _offsets(rows):
    return np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)


def _check_cover(rows, cap_rows, ncb):
    offs = _offsets(rows)
    units = B.moe_debug_gemm_units(offs, cap_rows, ncb)
    cover = np.zeros((max(int(offs[-1]), 1), ncb), dtype=np.int32)
    n_tiles = 0
    for h, e, row0, row_end, nb in units.tolist():
        if h == 0:
            continue
        assert h in (256, 128, 64)
        assert 0 <= e < len(rows) and 0 <= nb < ncb
        assert offs[e] <= row0 < row_end == offs[e + 1]
        cover[row0:min(row0 + h, row_end), nb] += 1
        n_tiles += 1
    assert (cover[:int(offs[-1])] == 1).all()
    return units, n_tiles


def test_tiles_cover_every_row_once_random_routings():
    rng = np.random.default_rng(1234)
    for trial in range(120):
        n_local = int(rng.integers(1, 17))
        ncb = int(rng.integers(1, 9))
        kind = trial % 4
        if kind == 0:    # anything, including empty experts
            rows = rng.integers(0, 700, n_local) * (rng.random(n_local) < 0.8)
        elif kind == 1:  # just around the block heights
            rows = rng.choice([63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 449, 512], n_local)
        elif kind == 2:  # multinomial as routing gives
            rows = rng.multinomial(int(rng.integers(1, 6000)), rng.dirichlet(np.ones(n_local)))
        else:            # a few rows per expert only
            rows = rng.integers(0, 40, n_local)
        rows = rows.astype(np.int64)
        cap = int(rows.sum()) + int(rng.integers(0, 300))
        _check_cover(rows, cap, ncb)


def test_empty_routing_and_single_row():
    units, n = _check_cover(np.zeros(8, dtype=np.int64), 0, 4)
    assert n == 0 and (units[:, 0] == 0).all()
    units, n = _check_cover(np.array([0, 0, 1, 0]), 1, 3)
    assert n == 3 and sorted(int(r[0]) for r in units if r[0]) == [64, 64, 64]


def test_remainder_tiles_and_padding():
    # a remainder of up to 64 / up to 128 rows is a 64- / 128-row tile; a larger one is padded to a
    # 256-row tile when the expert has a 256-row block to share the weights with (a second
    # remainder tile would stream them a second time), and is 128 + 64 rows up to 192 otherwise
    for rows in range(1, 1200):
        units, _ = _check_cover(np.array([rows]), rows, 1)
        h = units[:, 0][units[:, 0] > 0]
        r = rows % 256
        pad = 128 if rows >= 256 else 192
        assert (h == 64).sum() == (0 < r <= 64 or 128 < r <= pad)
        assert (h == 128).sum() == (64 < r <= pad)
        assert (h == 256).sum() == rows // 256 + (r > pad)
        assert h.sum() - rows < (64 if r <= pad else 128)


def test_experts_below_256_rows_are_padded_only_in_launches_that_fill_the_chip():
    rows = np.array([150, 190, 130, 100, 60, 193, 170, 129])
    few, _ = _check_cover(rows, int(rows.sum()), 2)       # 2 column blocks: 26 tiles in all
    many, _ = _check_cover(rows, int(rows.sum()), 112)    # 112 column blocks: 1456 tiles
    def heights(units, expert):
        return sorted(int(h) for h, e, _, _, nb in units if h and e == expert and nb == 0)
    for e, r in enumerate(rows):
        want_few = [256] if r > 192 else ([64, 128] if r > 128 else ([128] if r > 64 else [64]))
        want_many = [256] if r > 128 else ([128] if r > 64 else [64])
        assert heights(few, e) == want_few and heights(many, e) == want_many, (e, r)
    # the switch is at 256 tiles counted before any such padding
    rows = np.array([150] * 8)                            # 16 row blocks
    assert (np.asarray(_check_cover(rows, 1200, 15)[0])[:, 0] == 256).sum() == 0      # 240 tiles
    assert (np.asarray(_check_cover(rows, 1200, 16)[0])[:, 0] == 256).sum() == 8 * 16  # 256 tiles


def test_full_tiles_first_and_balanced_over_xcds():
    # 8 experts of about 1024 rows, 112 column blocks (the GEMM1 shape of an 8 x 14336 layer)
    rows = np.array([1040, 1030, 1050, 1024, 1000, 1047, 1033, 1025])
    units, _ = _check_cover(rows, int(rows.sum()), 112)
    per_xcd = []
    for x in range(8):   # workgroup b runs on XCD b % 8, in the order of b
        h = units[x::8, 0]
        h = h[h > 0]
        assert (np.diff(h) <= 0).all()          # 256-row tiles first, remainder tiles last
        per_xcd.append(((h == 256).sum(), (h == 64).sum()))
    full, small = zip(*per_xcd)
    assert max(full) - min(full) <= 1 and max(small) - min(small) <= 1
    # neighbours on one XCD share the weight panel: row blocks of one (expert, column block) are adjacent
    x0 = units[0::8]
    x0 = x0[x0[:, 0] == 256]
    same = (x0[1:, 1] == x0[:-1, 1]) & (x0[1:, 4] == x0[:-1, 4])
    assert same.mean() > 0.7


def test_invalid_arguments():
    L = B.lib()
    offs = np.array([0, 5, 3], dtype=np.int32)   # decreasing
    out = np.zeros((64, B.DEBUG_UNIT_INTS), dtype=np.int32)
    assert L.moe_debug_gemm_units(offs.ctypes.data, 2, 8, 1, out.ctypes.data, 64) == B.MOE_ERR_INVALID_ARG
    offs = np.array([0, 5, 9], dtype=np.int32)
    assert L.moe_debug_gemm_units(offs.ctypes.data, 2, 8, 1, out.ctypes.data, 64) == B.MOE_ERR_INVALID_ARG  # last > cap
    assert L.moe_debug_gemm_units(offs.ctypes.data, 2, 16, 1, out.ctypes.data, 2) == B.MOE_ERR_WORKSPACE


def _check_even_cover(rows, cap_rows, ncb):
    offs = _offsets(rows)
    units = B.moe_debug_even_units(offs, cap_rows, ncb)
    cover = np.zeros((max(int(offs[-1]), 1), ncb), dtype=np.int32)
    for h, e, row0, row_end, nb in units.tolist():
        if h == 0:
            continue
        assert h == 160 and 0 <= e < len(rows) and 0 <= nb < ncb
        assert offs[e] <= row0 < row_end == offs[e + 1] and (row0 - offs[e]) % 160 == 0
        cover[row0:min(row0 + h, row_end), nb] += 1
    assert (cover[:int(offs[-1])] == 1).all()
    return units


def test_even_row_blocks_cover_every_row_once():
    rng = np.random.default_rng(99)
    for trial in range(80):
        n_local = int(rng.integers(1, 70))
        ncb = int(rng.integers(1, 9))
        if trial % 3 == 0:
            rows = rng.integers(0, 700, n_local) * (rng.random(n_local) < 0.8)
        elif trial % 3 == 1:
            rows = rng.choice([1, 159, 160, 161, 319, 320, 321, 480, 481], n_local)
        else:
            rows = rng.multinomial(int(rng.integers(1, 20000)), rng.dirichlet(np.ones(n_local)))
        rows = rows.astype(np.int64)
        _check_even_cover(rows, int(rows.sum()) + int(rng.integers(0, 300)), ncb)
    units = _check_even_cover(np.zeros(5, dtype=np.int64), 0, 3)
    assert (units[:, 0] == 0).all()


def test_even_row_blocks_of_one_column_block_are_neighbours_on_one_xcd():
    # 60 experts of 250 to 300 rows, 11 column blocks (the gate/up projection of a 60 x 1408 layer at
    # 4096 tokens): the two row blocks of an (expert, column block) run side by side on one XCD, so
    # the second reader of the weight panel finds it in that XCD's L2
    rng = np.random.default_rng(3)
    rows = rng.integers(250, 301, 60)
    units = _check_even_cover(rows, int(rows.sum()), 11)
    assert (units[:, 0] == 160).sum() == 60 * 11 * 2
    pairs = same = 0
    for x in range(8):
        u = units[x::8]
        u = u[u[:, 0] > 0]
        for a, b in zip(u[:-1], u[1:]):
            if a[2] != b[2] and a[1] == b[1] and a[4] == b[4]:
                same += 1
        pairs += len(u) // 2
    assert same >= 0.95 * pairs


def test_tile_rows_rule():
    qwen = B.make_shard(60, 60, 0, 2048, 1408, 1408)
    # rows per expert just below one or two blocks of 160 rows
    assert B.moe_debug_tile_rows(4096 * 4, qwen) == 160      # 273 rows per expert
    assert B.moe_debug_tile_rows(2048 * 4, qwen) == 160      # 137
    assert B.moe_debug_tile_rows(3072 * 4, qwen) == 256      # 205: a second block for most experts, nothing saved
    assert B.moe_debug_tile_rows(1536 * 4, qwen) == 256      # 102
    assert B.moe_debug_tile_rows(8192 * 4, qwen) == 256      # 546
    assert B.moe_debug_tile_rows(4096 * 4, B.make_shard(60, 30, 0, 2048, 1408, 1408)) == 256   # 30 local experts
    assert B.moe_debug_tile_rows(4096 * 2, B.make_shard(8, 8, 0, 4096, 14336, 14336)) == 256   # 1024 rows per expert
    assert B.lib().moe_debug_tile_rows(-1, ctypes.byref(qwen)) == B.MOE_ERR_INVALID_ARG
    assert B.lib().moe_debug_tile_rows(-1, None) == B.MOE_ERR_INVALID_ARG
