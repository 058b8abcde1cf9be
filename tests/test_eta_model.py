"""Compute-simulation model (paper Sec. III-B): T_cal = F_module / Max_FLOPs * eta with eta from a
random forest on polynomial features, fitted on the measured Expert-module latency table."""
import os

import numpy as np

from paper_2508_19373_amd import eta_model as M
from paper_2508_19373_amd import inputs as I
from paper_2508_19373_amd.latency_table import legal_shards

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TABLE = os.path.join(ROOT, "profiles", "expert_latency_table_mi355x.csv")


def _row(T, tp=1, ep=1, model=I.MIXTRAL):
    return dict(model=model.name, hidden=model.hidden, n_experts=model.n_experts, top_k=model.top_k,
                inter=model.inter, inter_shared=model.inter_shared, tp=tp, ep=ep, ep_rank=0, tokens=T)


def test_legal_shards_follow_the_search_space_rules():
    mix = legal_shards(I.MIXTRAL)
    assert (1, 1) in mix and (8, 1) in mix and (1, 8) in mix and (2, 4) in mix
    assert all(tp * ep <= 8 and tp in (1, 2, 4, 8) and 8 % ep == 0 for tp, ep in mix)
    qw = legal_shards(I.QWEN)
    assert (1, 8) not in qw          # 8 does not divide 60 experts
    assert all(60 % ep == 0 and 1408 % tp == 0 for tp, ep in qw)


def test_module_flops_matches_hand_count():
    r = _row(4096)
    # router 2*T*H*E + routed 6*(T*k)*H*I
    want = 2 * 4096 * 4096 * 8 + 6 * 8192 * 4096 * 14336
    assert M.module_flops(r) == want
    q = _row(32, model=I.QWEN)
    want = 2 * 32 * 2048 * 60 + 6 * 128 * 2048 * 1408 + 6 * 32 * 2048 * 5632 + 2 * 32 * 2048
    assert M.module_flops(q) == want
    assert M.module_flops(_row(4096, tp=4)) < M.module_flops(r) / 3.9  # TP slices the expert FLOPs


def test_roofline_eta_regimes():
    assert M.roofline_eta(_row(8192)) == 1.0                     # prefill: compute-bound
    dec = _row(16)
    want = (M.weight_bytes(dec) / M.PEAK_BYTES) / (M.module_flops(dec) / M.PEAK_FLOPS)
    assert want > 50 and abs(M.roofline_eta(dec) - want) < 1e-9  # decode: memory-bound by weight loading


def test_recovers_a_synthetic_latency_law():
    rng = np.random.default_rng(0)
    rows = []
    for model in (I.MIXTRAL, I.QWEN):
        for tp, ep in legal_shards(model):
            for T in (16, 32, 64, 128, 256, 512, 1024, 2048, 4096, 8192):
                r = _row(T, tp, ep, model)
                t = max(M.module_flops(r) / (0.45 * M.PEAK_FLOPS), M.weight_bytes(r) / (0.7 * M.PEAK_BYTES)) + 25e-6
                r["us_per_layer"] = t * 1e6 * (1 + 0.02 * rng.standard_normal())
                rows.append(r)
    mean, mx, n = M.holdout_error(rows, seed=1, n_estimators=80)
    assert n >= 30 and mean < 0.08
    model = M.fit(rows, n_estimators=80)
    # the model is the paper's formula: T_cal = F / Max_FLOPs * eta
    sub = rows[:5]
    t = model.predict_us(sub)
    f = np.array([M.module_flops(r) for r in sub])
    assert np.allclose(t, f / M.PEAK_FLOPS * model.eta(sub) * 1e6)
    assert np.all(model.eta(sub) >= 1.0)


def test_measured_table_holdout_error_below_ten_percent():
    rows = M.load_table(TABLE)
    assert len(rows) >= 250
    errs = [M.holdout_error(rows, seed=s, n_estimators=100)[0] for s in range(3)]
    assert np.mean(errs) < 0.10, errs  # the paper reports < 10 % for its compute model
    # the table shows the two regimes the paper describes: flat latency at decode sizes,
    # growing with tokens at prefill sizes
    mix = {r["tokens"]: r["us_per_layer"] for r in rows if r["model"] == I.MIXTRAL.name and r["tp"] == 1 and r["ep"] == 1}
    assert mix[64] < 1.1 * mix[16] and mix[8192] > 1.6 * mix[4096]


def test_unmeasured_shard_is_predicted_from_the_measured_ones():
    # what the simulator is for: the latency of a configuration that was not measured.  Leave one
    # (model, E_t, E_e) shard out at a time, all its token counts and routings, fit on the rest.
    rows = M.load_table(TABLE)
    by_shard = M.group_holdout_error(rows, lambda r: (r["model"], r["tp"], r["ep"]), n_estimators=40)
    assert len(by_shard) == 29
    means = np.array([v[0] for v in by_shard.values()])
    print("leave-one-shard-out: mean of shard means %.3f, worst shard mean %.3f, largest single error %.3f"
          % (means.mean(), means.max(), max(v[1] for v in by_shard.values())))
    assert means.mean() < 0.12          # measured 0.096; the paper reports < 10 % for its compute model
    assert np.median(means) < 0.10
    # the miss is stated, not hidden: the shards at the edge of the grid (Qwen1.5 with its intermediate
    # size cut in 8, a slice of 176 zero-padded to 192) are off by 30 % on average
    assert means.max() < 0.45


def test_skewed_rows_use_the_rows_the_shard_receives():
    rows = M.load_table(TABLE)
    skew = [r for r in rows if r["routing"] == "zipf"]
    assert len(skew) >= 150 and {r["ep_rank"] for r in skew} >= {0.0, 1.0, 3.0}
    hot = [r for r in skew if r["model"] == I.MIXTRAL.name and r["tp"] == 1 and r["ep"] == 4 and r["ep_rank"] == 0 and r["tokens"] == 8192][0]
    cold = [r for r in skew if r["model"] == I.MIXTRAL.name and r["tp"] == 1 and r["ep"] == 4 and r["ep_rank"] == 3 and r["tokens"] == 8192][0]
    assert hot["routed_rows"] > 0.5 * 2 * 8192 and cold["routed_rows"] < 0.15 * 2 * 8192
    assert M.expected_rows(hot) == hot["routed_rows"] and M.module_flops(hot) > 5 * M.module_flops(cold)
    assert hot["us_per_layer"] > 3 * cold["us_per_layer"]          # the load imbalance the paper describes
    bal = dict(hot, routing="balanced")
    assert M.expected_rows(bal) == 8192 * 2 / 4
