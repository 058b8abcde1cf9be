"""Host logic around the V_dequant -> T_dequant dictionary (CPU only)."""
import os

import pytest

from paper_2508_19373_amd import dequant_table as D
from paper_2508_19373_amd import inputs as I

TABLE = os.path.join(os.path.dirname(__file__), "..", "profiles", "int4_dequant_table_mi355x.csv")


def test_expert_parameter_counts():
    # Mixtral-8x7B: 8 experts x 3 matrices x 14336 x 4096 per layer
    assert D.expert_params_per_layer(I.MIXTRAL) == 8 * 3 * 14336 * 4096
    assert D.expert_params_per_layer(I.QWEN) == 3 * 2048 * (60 * 1408 + 5632)
    for label, v in D.sizes():
        assert v % 64 == 0 and v > 0


def test_lookup_interpolates_and_extrapolates():
    table = [dict(v_dequant=100, us=10.0), dict(v_dequant=300, us=30.0), dict(v_dequant=200, us=20.0)]
    assert D.lookup(table, 150) == pytest.approx(15.0)
    assert D.lookup(table, 300) == pytest.approx(30.0)
    assert D.lookup(table, 50) == pytest.approx(10.0)       # below the table: the launch floor
    assert D.lookup(table, 400) == pytest.approx(40.0)      # above: the last slope


def test_measured_table_is_bandwidth_bound_and_linear():
    rows = D.load(TABLE)
    big = [r for r in rows if int(r["v_dequant"]) >= 1 << 27]
    assert len(big) >= 8
    for r in big:   # large transfers run at 70 % of the 8 TB/s HBM peak or better
        assert float(r["pct_hbm_peak"]) >= 70.0
    # T_dequant scales with V_dequant (the paper's premise for keying the dictionary on V)
    t1 = D.lookup(rows, 1 << 28)
    t2 = D.lookup(rows, 1 << 29)
    assert t2 / t1 == pytest.approx(2.0, rel=0.05)
    # a device of an 8-way expert-parallel Mixtral dequantises one eighth of a layer's expert weights
    v = D.expert_params_per_layer(I.MIXTRAL) // 8
    assert D.lookup(rows, v) == pytest.approx(v * D.BYTES_PER_WEIGHT / 6.3e6, rel=0.1)   # ~6.3 TB/s
