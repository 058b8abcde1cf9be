"""Strategy enumeration and exact search (CPU): the enumerations against hand counts, the search
against an independent ILP solver (scipy's HiGHS) on the paper's one-hot formulation, the switching
cost against its formula's special cases, and the memory bound."""
import math
import os

import numpy as np
import pytest
import scipy.optimize as so

from paper_2508_19373_amd import dequant_table as D
from paper_2508_19373_amd import strategy_search as S

PROFILES = os.path.join(os.path.dirname(__file__), "..", "profiles")


def test_attention_strategies_follow_head_divisibility():
    assert S.attention_strategies(S.MIXTRAL_8X7B, 8) == [(1, 8), (2, 4), (4, 2), (8, 1)]
    assert S.attention_strategies(S.QWEN15_MOE, 8) == [(1, 8), (2, 4), (4, 2), (8, 1)]
    assert S.attention_strategies(S.QWEN2_57B, 8) == [(1, 8), (2, 4), (4, 2)]   # 4 KV heads, 28 query heads
    assert S.attention_strategies(S.MIXTRAL_8X7B, 4) == [(1, 4), (2, 2), (4, 1)]


def test_expert_strategies_follow_the_ilp_constraints():
    # no DP for experts: E_t * E_e = N; E_t = 2^n divides the intermediate size; E_e divides the expert count
    assert S.expert_strategies(S.MIXTRAL_8X7B, 8) == [(1, 8), (2, 4), (4, 2), (8, 1)]
    assert S.expert_strategies(S.QWEN15_MOE, 8) == [(2, 4), (4, 2), (8, 1)]        # 8 does not divide 60
    assert S.expert_strategies(S.QWEN2_57B, 8) == [(1, 8), (2, 4), (4, 2), (8, 1)]
    for m in S.MODELS.values():
        for t, e in S.expert_strategies(m, 8):
            assert t * e == 8 and m.inter % t == 0 and m.n_experts % e == 0 and t & (t - 1) == 0


def _milp(n_layers, s_out, pre, dec, sw):
    """One binary per (k, i, j) triple with exactly one selected: the paper's one-hot S_k, E_i, E_j
    are its marginals."""
    ka, ke = len(pre), len(pre[0])
    c = np.array([n_layers * (pre[k][i] + s_out * dec[k][j]) + sw[k][i][j]
                  for k in range(ka) for i in range(ke) for j in range(ke)])
    res = so.milp(c, integrality=np.ones_like(c), bounds=so.Bounds(0, 1),
                  constraints=so.LinearConstraint(np.ones((1, c.size)), 1, 1))
    assert res.success
    return res.fun, int(np.argmax(res.x))


def test_exact_search_matches_an_ilp_solver_on_random_costs():
    rng = np.random.default_rng(0)
    for trial in range(30):
        ka, ke = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        pre = rng.uniform(1, 10, (ka, ke)).tolist()
        dec = rng.uniform(0.1, 1, (ka, ke)).tolist()
        sw = rng.uniform(0, 50, (ka, ke, ke))
        sw[:, np.arange(ke), np.arange(ke)] = 0
        s_out, n_layers = int(rng.integers(1, 300)), int(rng.integers(1, 40))
        (k, i, j), best = S.exact_search(n_layers, s_out, pre, dec, sw.tolist())
        ref, flat = _milp(n_layers, s_out, pre, dec, sw.tolist())
        assert best == pytest.approx(ref, rel=1e-12)
        assert (k * ke + i) * ke + j == flat or best == pytest.approx(
            n_layers * (pre[flat // (ke * ke)][(flat // ke) % ke] + s_out * dec[flat // (ke * ke)][flat % ke])
            + sw[flat // (ke * ke)][(flat // ke) % ke][flat % ke], rel=1e-12)


def test_exact_search_limits():
    pre = [[5.0, 1.0, 3.0]]
    dec = [[1.0, 3.0, 2.0]]
    free = [[[0.0] * 3 for _ in range(3)]]
    # free switching: prefill and decoding choose independently
    assert S.exact_search(2, 10, pre, dec, free)[0] == (0, 1, 0)
    # prohibitive switching: the same strategy in both stages, the best compromise
    wall = [[[0.0 if i == j else 1e9 for j in range(3)] for i in range(3)]]
    (k, i, j), v = S.exact_search(2, 10, pre, dec, wall)
    assert i == j == 0 and v == pytest.approx(2 * (5 + 10 * 1))
    # one generated token: the prefill optimum wins
    assert S.exact_search(2, 1, pre, dec, wall)[0] == (0, 1, 1)


def test_switching_cost_formula_cases():
    hw = S.Hardware()
    m = S.MIXTRAL_8X7B
    rows = D.load(os.path.join(PROFILES, "int4_dequant_table_mi355x.csv"))
    same = S.switching_seconds(m, hw, (8, 1), (8, 1), 0.0, rows)
    assert same == 0.0
    v = m.expert_params_per_layer // 8
    t_up = v * D.BYTES_PER_WEIGHT_IN / hw.pcie_bw
    t_dq = D.lookup(rows, v) * 1e-6
    t_rs = hw.coll_latency + (v * 2.0 / 8) / hw.link_bw * 7
    # nothing to hide behind: min{reshard, upload + dequant}
    assert S.switching_seconds(m, hw, (1, 8), (8, 1), 0.0, rows) == pytest.approx(m.n_layers * min(t_rs, t_up + t_dq))
    # a prefill layer longer than upload + dequant hides the whole transition
    assert S.switching_seconds(m, hw, (1, 8), (8, 1), 10.0, rows) == 0.0
    # partial overlap
    half = 0.5 * (t_up + t_dq)
    assert S.switching_seconds(m, hw, (1, 8), (8, 1), half, rows) == pytest.approx(m.n_layers * min(t_rs, half))


def test_memory_bound_prunes_data_parallel_attention():
    m = S.MIXTRAL_8X7B
    sc = S.Scenario(batch=8, s_in=4096, s_out=2048)
    roomy = S.Hardware()
    assert all(S.memory_ok(m, roomy, sc, a) for a in S.attention_strategies(m, 8))
    # per device: KV cache 0.81 GB + expert weights 11.27 GB for every strategy; attention weights
    # 0.34 GB per replica (A_d of them); activations 2 * 0.134 GB per sequence of the micro-batch
    # (8 / A_d of them):  (1,8) 15.03 GB, (2,4) 13.96 GB, (4,2) 13.82 GB, (8,1) 14.56 GB
    tight = S.Hardware(mem_bytes=14.2e9)
    ok = [a for a in S.attention_strategies(m, 8) if S.memory_ok(m, tight, sc, a)]
    assert ok == [(2, 4), (4, 2)]   # eight attention replicas and an eight-sequence micro-batch are both too big
    assert not any(S.memory_ok(m, S.Hardware(mem_bytes=1e9), sc, a) for a in S.attention_strategies(m, 8))
    with pytest.raises(ValueError):
        S.search(m, sc, hw=S.Hardware(mem_bytes=1e9))


def test_search_on_the_measured_tables_beats_or_ties_tp_everywhere():
    t_e = S.ExpertLatencyTable()
    for m in S.MODELS.values():
        for s_in, s_out in ((256, 64), (4096, 64), (4096, 2048)):
            sc = S.Scenario(batch=8, s_in=s_in, s_out=s_out)
            c = S.search(m, sc, t_e=t_e)
            assert c.attention in S.attention_strategies(m, 8)
            assert c.expert_prefill in S.expert_strategies(m, 8) and c.expert_decode in S.expert_strategies(m, 8)
            assert c.total_s == pytest.approx(c.prefill_s + c.decode_s + c.switch_s)
            assert c.total_s <= S.tp_baseline(m, sc, t_e=t_e) * (1 + 1e-12)


def test_latency_table_interpolation_is_log_log():
    t_e = S.ExpertLatencyTable()
    key = ("mixtral-8x7b", 1, 1)
    pts = t_e.curves[key]
    (x0, y0), (x1, y1) = pts[3], pts[4]
    mid = math.exp(0.5 * (x0 + x1))
    assert t_e.seconds(*key, mid) == pytest.approx(math.exp(0.5 * (y0 + y1)) * 1e-6)
    assert t_e.seconds(*key, math.exp(x1)) == pytest.approx(math.exp(y1) * 1e-6)
    assert t_e.seconds(*key, 1) == pytest.approx(math.exp(pts[0][1]) * 1e-6)
