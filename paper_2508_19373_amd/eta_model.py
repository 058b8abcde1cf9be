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
            if k not in ("model", "launch_mode"):
                r[k] = float(v)
    return rows


def features_of(row) -> np.ndarray:
    tp, ep = row["tp"], row["ep"]
    vals = dict(tokens=row["tokens"], hidden=row["hidden"], inter_slice=row["inter"] / tp,
                n_local_experts=row["n_experts"] / ep, top_k=row["top_k"], n_experts=row["n_experts"],
                inter_shared_slice=row["inter_shared"] / tp)
    # derived from the same parameters: expected rows per local expert (decides the regime), the
    # module's FLOPs and the bytes of weights it touches (their ratio is the arithmetic intensity)
    vals["rows_per_expert"] = row["tokens"] * row["top_k"] / row["n_experts"]
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


def module_flops(row) -> float:
    """F_module: algorithmic FLOPs of the shard's Expert module, expected routed rows."""
    T, H, E, k = row["tokens"], row["hidden"], row["n_experts"], row["top_k"]
    I_s, I_sh = row["inter"] / row["tp"], row["inter_shared"] / row["tp"]
    rows = T * k / row["ep"]  # expected routed rows of the shard (known before the run)
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
