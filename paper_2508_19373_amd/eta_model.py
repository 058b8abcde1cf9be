"""Compute-simulation model of the Expert module (paper, Sec. III-B "Inference Latency Estimation"):

    T_cal = F_module / Max_FLOPs * eta

with eta fitted by a random-forest regressor on a polynomial expansion of the request and model
parameters (the paper names b, s, h; here the token count T = b*s reaches the Expert module, and
the shard dimensions are added because one table covers several models and strategies).  The
training set is the measured operator-latency table written by latency_table.py.  CPU only.
"""
from __future__ import annotations

import csv
from dataclasses import dataclass

import numpy as np

PEAK_FLOPS = 2.5e15  # MI355X dense bf16 MFMA, FLOP/s
PEAK_BYTES = 8.0e12  # MI355X HBM3E, B/s

FEATURES = ("tokens", "hidden", "inter_slice", "n_local_experts", "top_k", "n_experts", "inter_shared_slice",
            "rows_per_expert", "flops", "weight_bytes")


def load_table(path):
    with open(path) as f:
        rows = list(csv.DictReader(f))
    for r in rows:
        for k, v in r.items():
            if k not in ("model", "launch_mode", "routing"):
                r[k] = float(v)
        r.setdefault("routing", "balanced")
    return rows


def features_of(row) -> np.ndarray:
    tp, ep = row["tp"], row["ep"]
    vals = dict(tokens=row["tokens"], hidden=row["hidden"], inter_slice=row["inter"] / tp,
                n_local_experts=row["n_experts"] / ep, top_k=row["top_k"], n_experts=row["n_experts"],
                inter_shared_slice=row["inter_shared"] / tp)
    # derived from the same parameters: expected rows per local expert (decides the regime), the
    # module's FLOPs and the bytes of weights it touches (their ratio is the arithmetic intensity)
    vals["rows_per_expert"] = expected_rows(row) / (row["n_experts"] / ep)
    vals["flops"] = module_flops(row)
    vals["weight_bytes"] = weight_bytes(row)
    return np.log2(np.maximum(np.array([vals[k] for k in FEATURES], dtype=np.float64), 1.0))


def weight_bytes(row) -> float:
    """Bytes of expert weights the shard has to read: 3*H*I_s*2 per expected active local expert
    plus the shared expert."""
    n_loc = row["n_experts"] / row["ep"]
    active = n_loc * (1.0 - (1.0 - row["top_k"] / row["n_experts"]) ** row["tokens"])
    return 6.0 * row["hidden"] * (active * row["inter"] / row["tp"] + row["inter_shared"] / row["tp"])


def roofline_eta(row, peak_flops=PEAK_FLOPS) -> float:
    """eta of a kernel that sits exactly on the roofline: max(1, memory time / compute time)."""
    return max(1.0, (weight_bytes(row) / PEAK_BYTES) / (module_flops(row) / peak_flops))


def expected_rows(row) -> float:
    """Routed rows of the shard, known before the run: its balanced share T*k/E_e, or, under a
    skewed expert popularity, the share that popularity gives the shard's experts (the table
    records it in `routed_rows`; a simulator would compute it from the popularity it assumes)."""
    if row.get("routing", "balanced") != "balanced" and "routed_rows" in row:
        return float(row["routed_rows"])
    return row["tokens"] * row["top_k"] / row["ep"]


def module_flops(row) -> float:
    """F_module: algorithmic FLOPs of the shard's Expert module, expected routed rows."""
    T, H, E, k = row["tokens"], row["hidden"], row["n_experts"], row["top_k"]
    I_s, I_sh = row["inter"] / row["tp"], row["inter_shared"] / row["tp"]
    rows = expected_rows(row)
    return 2.0 * T * H * E + 6.0 * rows * H * I_s + (6.0 * T * H * I_sh + 2.0 * T * H if I_sh else 0.0)


@dataclass
class EtaModel:
    poly: object
    forest: object
    peak_flops: float = PEAK_FLOPS

    def eta(self, rows) -> np.ndarray:
        X = np.stack([features_of(r) for r in rows])
        base = np.array([roofline_eta(r, self.peak_flops) for r in rows])
        return base * np.exp2(self.forest.predict(self.poly.transform(X)))

    def predict_us(self, rows) -> np.ndarray:
        f = np.array([module_flops(r) for r in rows])
        return f / self.peak_flops * self.eta(rows) * 1e6


def fit(rows, *, degree=2, n_estimators=200, seed=0, peak_flops=PEAK_FLOPS) -> EtaModel:
    """eta = T_measured / (F_module / Max_FLOPs).  eta spans three orders of magnitude between decode
    and prefill, almost all of it the memory/compute ratio of the roofline, which is known in closed
    form; the forest is fitted on log2(eta / roofline_eta), a quantity of order one, so that its
    piecewise-constant prediction interpolates well between the measured token counts."""
    from sklearn.ensemble import RandomForestRegressor
    from sklearn.preprocessing import PolynomialFeatures
    X = np.stack([features_of(r) for r in rows])
    f = np.array([module_flops(r) for r in rows])
    t = np.array([r["us_per_layer"] for r in rows]) * 1e-6
    eta = t / (f / peak_flops)
    poly = PolynomialFeatures(degree=degree, include_bias=False).fit(X)
    forest = RandomForestRegressor(n_estimators=n_estimators, random_state=seed, min_samples_leaf=1)
    base = np.array([roofline_eta(r, peak_flops) for r in rows])
    forest.fit(poly.transform(X), np.log2(eta / base))
    return EtaModel(poly, forest, peak_flops)


def holdout_error(rows, *, test_fraction=0.2, seed=0, **kw):
    """Relative error |T_pred - T_meas| / T_meas on a random hold-out; returns (mean, max, n_test)."""
    rng = np.random.default_rng(seed)
    idx = rng.permutation(len(rows))
    n_test = max(1, int(round(test_fraction * len(rows))))
    test, train = [rows[i] for i in idx[:n_test]], [rows[i] for i in idx[n_test:]]
    model = fit(train, seed=seed, **kw)
    pred = model.predict_us(test)
    meas = np.array([r["us_per_layer"] for r in test])
    err = np.abs(pred - meas) / meas
    return float(err.mean()), float(err.max()), n_test


def group_holdout_error(rows, key, **kw):
    """Leave-one-group-out: for every value of `key(row)` fit on all other rows and predict that
    group's.  Returns {group: (mean relative error, max relative error, n)}.  With key = the shard
    (model, E_t, E_e) this asks what the paper's simulator is for: the latency of a configuration
    that was not measured, from those that were; with key = the model, a model never seen."""
    groups = {}
    for i, r in enumerate(rows):
        groups.setdefault(key(r), []).append(i)
    out = {}
    for g, idx in groups.items():
        held = set(idx)
        train = [r for i, r in enumerate(rows) if i not in held]
        test = [rows[i] for i in idx]
        model = fit(train, **kw)
        pred = model.predict_us(test)
        meas = np.array([r["us_per_layer"] for r in test])
        err = np.abs(pred - meas) / meas
        out[g] = (float(err.mean()), float(err.max()), len(idx))
    return out


def report(path):
    """Hold-out errors of the table at `path`, as text (what the design doc quotes)."""
    rows = load_table(path)
    lines = ["%d rows" % len(rows)]
    rnd = [holdout_error(rows, seed=s, n_estimators=100) for s in range(6)]
    lines.append("random 20 %% hold-out, 6 splits: mean %.1f %% (%.1f-%.1f), max %.1f %%"
                 % (100 * np.mean([r[0] for r in rnd]), 100 * min(r[0] for r in rnd), 100 * max(r[0] for r in rnd),
                    100 * max(r[1] for r in rnd)))
    by_shard = group_holdout_error(rows, lambda r: (r["model"], r["tp"], r["ep"]), n_estimators=60)
    means = [v[0] for v in by_shard.values()]
    worst = max(by_shard.items(), key=lambda kv: kv[1][0])
    lines.append("leave-one-shard-out, %d shards: mean of shard means %.1f %%, worst shard %s mean %.1f %% max %.1f %%, "
                 "largest single error %.1f %%" % (len(by_shard), 100 * np.mean(means), worst[0], 100 * worst[1][0],
                                                   100 * worst[1][1], 100 * max(v[1] for v in by_shard.values())))
    by_model = group_holdout_error(rows, lambda r: r["model"], n_estimators=60)
    for m, (mean, mx, n) in by_model.items():
        lines.append("leave-one-model-out, %s (%d rows): mean %.1f %%, max %.1f %%" % (m, n, 100 * mean, 100 * mx))
    return "\n".join(lines)


if __name__ == "__main__":
    import sys
    print(report(sys.argv[1]))
