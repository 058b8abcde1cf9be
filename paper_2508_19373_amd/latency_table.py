"""Operator benchmarking protocol for the Expert module: sweep (model shape, TP/EP shard, tokens)
on the GPU and write the measured per-layer latency table T_e that the compute-simulation model
is fitted on (paper, Sec. III-B "Inference Latency Estimation": the regressors' training sets
are measured operator latencies; Sec. III-C: T_e is the Expert module's cost vector over the
strategies of the search space, TP degree a power of two, EP degree dividing the expert count).

    python -m paper_2508_19373_amd.latency_table --out profiles/expert_latency_table_mi355x.csv
"""
from __future__ import annotations

import argparse
import csv
import sys
import time

FIELDS = ["model", "hidden", "n_experts", "top_k", "inter", "inter_shared", "tp", "ep", "ep_rank", "routing", "tokens",
          "routed_rows", "active_experts", "flops", "weight_bytes", "us_per_layer", "launch_mode"]

DEFAULT_TOKENS = (16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 1536, 2048, 3072, 4096, 6144, 8192)
# Expert-parallel shards are also measured under skewed routing (Zipf(1.2) expert popularity: the load
# imbalance the paper names as expert parallelism's weakness), on the shard that holds the most
# popular experts (rank 0) and the one that holds the least popular (last rank), at fewer token counts.
SKEWED_TOKENS = (16, 64, 256, 1024, 4096, 8192)


def legal_shards(shape, max_devices=8):
    """(E_t, E_e) with E_t a power of two dividing I, E_e dividing E, E_t * E_e <= max_devices, and
    no triple hybrid (the paper excludes DP for experts).  Slices that are not a multiple of 64 are
    zero-padded by the layer."""
    out = []
    for tp in (1, 2, 4, 8):
        for ep in (1, 2, 4, 8):
            if tp * ep > max_devices or shape.n_experts % ep or shape.inter % tp:
                continue
            if shape.inter_shared % tp:
                continue
            out.append((tp, ep))
    return out


def weight_sets(layer, total_bytes=1 << 30):
    """The layer's weights plus as many device copies as it takes to exceed `total_bytes` in all."""
    def nbytes(ws):
        return sum(t.numel() * t.element_size() for t in ws[:3]) + \
            (sum(t.numel() * t.element_size() for t in ws[3]) if ws[3] is not None else 0)
    first = (layer.w_gate, layer.w_up, layer.w_down, layer.shared)
    sets = [first]
    one = max(nbytes(first), 1)
    while len(sets) * one < total_bytes and len(sets) < 16:
        sets.append((first[0].clone(), first[1].clone(), first[2].clone(),
                     None if first[3] is None else [t.clone() for t in first[3]]))
    return sets


def measure(shape, tokens, seed=0, steps=60, warmup=30):
    import numpy as np
    import torch
    from . import inputs as I
    from .layer import ExpertShardLayer, bf16_tensor
    from .work import algorithmic_work

    li = I.make_layer_inputs(shape, 1, seed)
    layer = ExpertShardLayer.from_inputs(li, max_tokens=max(tokens))
    rows = []
    for T in tokens:
        x = bf16_tensor(I.make_x(seed, T, shape.hidden))
        logits = None
        if shape.router == "zipf":
            logits = torch.from_numpy(I.make_zipf_logits(seed, T, shape.n_experts)).cuda()

        def timed(fn, batches=3):
            # median of three timed batches: a single batch of a 100 us layer lasts a few
            # milliseconds, and one in twenty of those came out 10-15 % off
            for _ in range(warmup):
                fn()
            out = []
            for _ in range(batches):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(steps):
                    fn()
                torch.cuda.synchronize()
                out.append((time.perf_counter() - t0) * 1e6 / steps)
            return sorted(out)[len(out) // 2]

        # a shard whose weights fit the last-level cache (256 MB) would be served from it when the same
        # buffers are replayed; in a model every layer has its own weights.  Rotate over copies
        # that together exceed 1 GB.
        sets = weight_sets(layer)

        def use(ws):
            layer.w_gate, layer.w_up, layer.w_down, layer.shared = ws

        def rotating(fns):
            state = {"i": 0}

            def run():
                fns[state["i"] % len(fns)]()
                state["i"] += 1
            return run

        def eager_on(ws):
            def run():
                use(ws)
                layer.forward(x, logits)
            return run

        us, mode = timed(rotating([eager_on(ws) for ws in sets])), "eager"
        if us < 1000.0:
            graphs = []
            for ws in sets:
                use(ws)
                graphs.append(layer.capture(x, logits)[0])
            us, mode = timed(rotating([g.replay for g in graphs])), "hip-graph"
            del graphs
        use(sets[0])
        counts = np.diff(layer.expert_offsets.cpu().numpy())
        flops, min_bytes, R, active = algorithmic_work(shape, T, counts)
        rows.append(dict(model=shape.name, hidden=shape.hidden, n_experts=shape.n_experts, top_k=shape.top_k,
                         inter=shape.inter, inter_shared=shape.inter_shared, tp=shape.tp_degree, ep=shape.ep_degree,
                         ep_rank=shape.ep_rank, routing="zipf" if shape.router == "zipf" else "balanced", tokens=T,
                         routed_rows=R, active_experts=active, flops=flops,
                         weight_bytes=min_bytes, us_per_layer=round(us, 2), launch_mode=mode))
        print(rows[-1], flush=True)
    del layer
    torch.cuda.empty_cache()
    return rows


def main():
    from . import inputs as I
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", required=True)
    ap.add_argument("--tokens", type=int, nargs="*", default=list(DEFAULT_TOKENS))
    ap.add_argument("--models", nargs="*", default=["mixtral", "qwen", "qwen2_57b"])
    ap.add_argument("--no-skew", action="store_true", help="balanced routing only")
    ap.add_argument("--shard", default=None,
                    help="MODEL:TP:EP[:EP_RANK[:zipf]], measure this one shard in this process")
    args = ap.parse_args()
    bases = {"mixtral": I.MIXTRAL, "qwen": I.QWEN, "qwen2_57b": I.QWEN2_57B}

    def write(rows):
        with open(args.out, "w", newline="") as f:
            w = csv.DictWriter(f, fieldnames=FIELDS)
            w.writeheader()
            w.writerows(rows)

    if args.shard is not None:
        from dataclasses import replace
        parts = args.shard.split(":")
        m, tp, ep = parts[0], int(parts[1]), int(parts[2])
        rank = int(parts[3]) if len(parts) > 3 else 0
        shape = bases[m].shard(tp_degree=tp, tp_rank=0, ep_degree=ep, ep_rank=rank)
        if len(parts) > 4 and parts[4] == "zipf":
            shape = replace(shape, router="zipf")
        write(measure(shape, args.tokens))
        return
    # One child process per shard (this one never touches the GPU).  In the memory-bound regime a
    # layer whose weights were allocated after a larger layer was freed, from torch's cache or anew,
    # measured 3-10 % slower than the same layer in a fresh process; a model is loaded once.
    import os
    import subprocess
    import tempfile
    rows = []
    for m in args.models:
        for tp, ep in legal_shards(bases[m]):
            jobs = [("%s:%d:%d" % (m, tp, ep), args.tokens)]
            if ep > 1 and not args.no_skew:
                skewed = [t for t in SKEWED_TOKENS if t <= max(args.tokens)]
                jobs += [("%s:%d:%d:%d:zipf" % (m, tp, ep, rank), skewed) for rank in (0, ep - 1)]
            for spec, tokens in jobs:
                with tempfile.TemporaryDirectory() as d:
                    part = os.path.join(d, "part.csv")
                    subprocess.run([sys.executable, "-m", "paper_2508_19373_amd.latency_table", "--out", part,
                                    "--shard", spec, "--tokens", *[str(t) for t in tokens]], check=True)
                    with open(part, newline="") as f:
                        rows += list(csv.DictReader(f))
    write(rows)
    print("wrote %d rows to %s" % (len(rows), args.out))


if __name__ == "__main__":
    main()
