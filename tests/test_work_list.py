"""Host logic of the prefill grouped GEMM: the per-workgroup work list, run on the CPU through
moe_debug_gemm_units.  For any routing, the tiles of all workgroups must cover every routed row of
every column block exactly once, never reach into another expert's rows, and the grid bound the
launcher uses must hold."""
import numpy as np
import pytest

from paper_2508_19373_amd import binding as B


def _offsets(rows):
    return np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)


def _check_cover(rows, cap_rows, ncb, group):
    offs = _offsets(rows)
    units = B.moe_debug_gemm_units(offs, cap_rows, ncb, group)
    cover = np.zeros((max(int(offs[-1]), 1), ncb), dtype=np.int32)
    n_tiles = 0
    for rec in units:
        h, n = int(rec[0]), int(rec[1])
        assert (h == 0) == (n == 0)
        assert n <= (1 if h == 256 else 3)
        for t in range(n):
            e, row0, row_end, nb = (int(v) for v in rec[2 + 4 * t: 6 + 4 * t])
            assert 0 <= e < len(rows) and 0 <= nb < ncb
            assert offs[e] <= row0 < row_end == offs[e + 1]
            cover[row0:min(row0 + h, row_end), nb] += 1
            n_tiles += 1
    assert (cover[:int(offs[-1])] == 1).all()
    return units, n_tiles


@pytest.mark.parametrize("group", [1, 3])
def test_units_cover_every_row_once_random_routings(group):
    rng = np.random.default_rng(1234 + group)
    for trial in range(60):
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
        _check_cover(rows, cap, ncb, group)


def test_units_empty_routing_and_single_row():
    units, n = _check_cover(np.zeros(8, dtype=np.int64), 0, 4, 1)
    assert n == 0 and (units[:, 1] == 0).all()
    units, n = _check_cover(np.array([0, 0, 1, 0]), 1, 3, 3)
    assert n == 3 and sorted(int(r[0]) for r in units if r[1]) == [64]


def test_grouped_small_tiles_are_spread_between_full_tiles():
    # 8 experts of 1024 + a short tail, 112 column blocks (the GEMM1 shape of an 8 x 14336 layer)
    rows = np.array([1040, 1030, 1050, 1024, 1000, 1047, 1033, 1025])
    units, _ = _check_cover(rows, int(rows.sum()), 112, 0)   # launcher's choice: grouped
    busy = units[units[:, 1] > 0]
    small = busy[busy[:, 0] == 64]
    assert len(small) > 0 and (small[:, 1] <= 3).all() and (small[:-8, 1].max() == 3)
    # per XCD (workgroup id mod 8) the small units are not bunched: between two of them lie full tiles
    for x in range(8):
        seq = units[x::8]
        seq = seq[seq[:, 1] > 0][:, 0]
        pos = np.flatnonzero(seq == 64)
        assert len(pos) >= 2 and np.diff(pos).min() >= 8
    # few-round launch (GEMM2 shape, 16 column blocks): one small tile per unit, all after the full ones
    units, _ = _check_cover(rows, int(rows.sum()), 16, 0)
    for x in range(8):
        seq = units[x::8]
        seq = seq[seq[:, 1] > 0]
        assert (seq[:, 1] == 1).all()
        h = seq[:, 0]
        assert (np.diff(h) <= 0).all()   # 256s first, then the remainder tiles


def test_invalid_arguments():
    L = B.lib()
    offs = np.array([0, 5, 3], dtype=np.int32)   # decreasing
    out = np.zeros((64, B.DEBUG_UNIT_INTS), dtype=np.int32)
    assert L.moe_debug_gemm_units(offs.ctypes.data, 2, 8, 1, 1, out.ctypes.data, 64) == B.MOE_ERR_INVALID_ARG
    offs = np.array([0, 5, 9], dtype=np.int32)
    assert L.moe_debug_gemm_units(offs.ctypes.data, 2, 8, 1, 1, out.ctypes.data, 64) == B.MOE_ERR_INVALID_ARG  # last > cap
    assert L.moe_debug_gemm_units(offs.ctypes.data, 2, 16, 1, 2, out.ctypes.data, 64) == B.MOE_ERR_INVALID_ARG  # group
    assert L.moe_debug_gemm_units(offs.ctypes.data, 2, 16, 1, 1, out.ctypes.data, 2) == B.MOE_ERR_WORKSPACE
