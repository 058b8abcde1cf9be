"""V_dequant -> T_dequant dictionary of the switching cost (paper, "The Dynamic Parallelism
Transition Strategy": the dequantisation overhead scales with the number of dequantised
parameters, which depends on the number of GPUs; a dictionary V_dequant -> T_dequant is built
and queried at run time).  This sweep measures moe_int4_dequantize on the GPU for the parameter
counts one device dequantises per layer when the Expert module of each model is spread over
N = 1, 2, 4, 8 devices, plus a geometric ladder of sizes, and writes the table.

    python -m paper_2508_19373_amd.dequant_table --out profiles/int4_dequant_table_mi355x.csv
"""
from __future__ import annotations

import argparse
import csv

FIELDS = ["label", "v_dequant", "us", "gbs", "pct_hbm_peak"]
BYTES_PER_WEIGHT_IN = 0.5 + 4.0 / 64              # codes + (scale, min) per 64 weights
BYTES_PER_WEIGHT = BYTES_PER_WEIGHT_IN + 2.0      # ... read, bf16 written
PEAK_HBM_GBS = 8000.0


def expert_params_per_layer(shape) -> int:
    """Routed plus shared expert weights of one layer (gate, up, down)."""
    return 3 * shape.hidden * (shape.n_experts * shape.inter + shape.inter_shared)


def sizes():
    from . import inputs as I
    out = []
    for shape in (I.MIXTRAL, I.QWEN, I.QWEN2_57B):
        for n in (1, 2, 4, 8):
            v = expert_params_per_layer(shape) // n
            out.append(("%s/N=%d" % (shape.name, n), v - v % 64))
    v = 1 << 16
    while v <= 1 << 31:
        out.append(("2^%d" % (v.bit_length() - 1), v))
        v <<= 1
    return out


def measure(v: int, steps=20, warmup=10):
    import torch
    from . import binding as B
    codes = torch.randint(0, 256, (v // 2,), dtype=torch.uint8, device="cuda")
    qp = torch.full((v // 64, 2), 0x3C00, dtype=torch.int16, device="cuda")
    out = torch.empty(v, dtype=torch.bfloat16, device="cuda")
    for _ in range(warmup):
        B.moe_int4_dequantize(codes, qp, v, out)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(steps):
        B.moe_int4_dequantize(codes, qp, v, out)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / steps


def lookup(table, v: int) -> float:
    """T_dequant (us) for v parameters: linear interpolation between the table's neighbours."""
    pts = sorted((int(r["v_dequant"]), float(r["us"])) for r in table)
    if v <= pts[0][0]:
        return pts[0][1]
    for (v0, t0), (v1, t1) in zip(pts, pts[1:]):
        if v <= v1:
            return t0 + (t1 - t0) * (v - v0) / max(v1 - v0, 1)
    (v0, t0), (v1, t1) = pts[-2], pts[-1]
    return t1 + (t1 - t0) * (v - v1) / max(v1 - v0, 1)


def load(path):
    with open(path) as f:
        return list(csv.DictReader(f))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    rows = []
    for label, v in sizes():
        us = measure(v)
        gbs = v * BYTES_PER_WEIGHT / us / 1e3
        rows.append(dict(label=label, v_dequant=v, us=round(us, 2), gbs=round(gbs, 1),
                         pct_hbm_peak=round(100 * gbs / PEAK_HBM_GBS, 1)))
        print(rows[-1], flush=True)
    with open(args.out, "w", newline="") as f:
        w = csv.DictWriter(f, fieldnames=FIELDS)
        w.writeheader()
        w.writerows(rows)


if __name__ == "__main__":
    main()
