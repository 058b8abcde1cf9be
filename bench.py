#!/usr/bin/env python3
"""Benchmark of the MoE Expert-module forward pass on one MI355X shard.

A step is one pass of the whole hot path (route -> permute -> grouped SwiGLU FFN
[-> shared expert] -> combine) over one batch of seeded synthetic input that is already
resident in HBM.  Prints ONE JSON line: whole-layer throughput in bf16 TFLOP/s (algorithmic
FLOPs only), ms per step, a roofline object for the dominant kernel measured live with
events on the launch stream, and the CPU oracle timed on a bounded sample of the same
workload.  The line's `also` object holds the same measurement (50 steps after 30) of the other
target shapes, taken in the same process: the Mixtral-sized decode batch, its tensor-parallel and
expert-parallel shards, and the Qwen-sized layer at prefill and decode sizes.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload mixtral_prefill] [--no-also]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E

# HBM-side bytes per launch of the dominant kernel (GEMM1 + SwiGLU), from two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE in KiB per dispatch; see profiles/<workload>_rocprofv3.txt), each scaled by
# what the same counter reads for a plain 1 GiB device copy: FETCH_SIZE x 2.0, WRITE_SIZE x 1.0.
MEASURED_TRAFFIC_BYTES = {
    "mixtral_prefill": (1958763.1 * 2.0 + 232963.1) * 1024,
    "mixtral_decode": (936763.1 * 2.0 + 898.7) * 1024,
    "qwen_prefill": (405805.6 * 2.0 + 45056.0) * 1024,
}

# measured after the main workload in the same run (`also` in the JSON line): the other target shapes
ALSO_WORKLOADS = ("mixtral_decode", "mixtral_tp4_prefill", "mixtral_tp4_decode", "mixtral_ep4_hot", "mixtral_ep4_cold",
                  "qwen_prefill", "qwen_decode")

# name -> (inputs.WORKLOADS key, token count, description)
WORKLOADS = {
    "tiny": ("tiny", 64, "tiny 512/8e/top2/1024 T=64"),
    "mixtral_prefill": ("mixtral", 4096, "mixtral-8x7b unsharded prefill T=4096"),
    "mixtral_decode": ("mixtral", 16, "mixtral-8x7b unsharded decode T=16"),
    "mixtral_tp4_prefill": ("mixtral_tp4", 8192, "mixtral-8x7b TP=4 shard T=8192"),
    "mixtral_tp4_decode": ("mixtral_tp4", 64, "mixtral-8x7b TP=4 shard T=64"),
    "mixtral_ep4_hot": ("mixtral_ep4_hot", 8192, "mixtral-8x7b EP=4 shard experts 0-1, Zipf(1.2), T=8192 global"),
    "mixtral_ep4_cold": ("mixtral_ep4_cold", 8192, "mixtral-8x7b EP=4 shard experts 6-7, Zipf(1.2), T=8192 global"),
    "qwen_prefill": ("qwen", 4096, "qwen1.5-moe-a2.7b + shared expert T=4096"),
    "qwen_decode": ("qwen", 32, "qwen1.5-moe-a2.7b + shared expert T=32"),
    "qwen2_57b_prefill": ("qwen2_57b", 4096, "qwen2-57b-a14b + shared expert T=4096"),
    "qwen2_57b_decode": ("qwen2_57b", 32, "qwen2-57b-a14b + shared expert T=32"),
}


from paper_2508_19373_amd.work import algorithmic_work  # noqa: E402


def time_events(fn, iters, torch):
    """Average duration (ms) of fn() over `iters` back-to-back launches, from events recorded
    on the stream the kernels are launched on (torch's current stream)."""
    start, end = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    end.record()
    end.synchronize()
    return start.elapsed_time(end) / iters


def measure(workload, steps, warmup, args, torch, np, B, I, ExpertShardLayer, bf16_tensor):
    """One workload: whole-layer time over `steps` steps after `warmup`, per-call breakdown, and
    the roofline of its dominant kernel.  Returns a dict of everything the JSON line needs."""
    key, T, desc = WORKLOADS[workload]
    shape, _ = I.WORKLOADS[key]
    t0 = time.time()
    li = I.make_layer_inputs(shape, T, args.seed)
    gen_s = time.time() - t0
    layer = ExpertShardLayer.from_inputs(li, overlap_shared=not args.no_overlap_shared,
                                         gather_in_ffn=False if args.permuted_copy else (True if args.gather_rows else None))
    x = bf16_tensor(li.x)
    logits = None if li.logits is None else torch.from_numpy(li.logits).cuda()

    def step():
        return layer.forward(x, logits)

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    eager_ms = timed(step)
    ms_per_step, mode = eager_ms, "eager"
    if args.graph == "on" or (args.graph == "auto" and eager_ms < 1.0):
        graph, _ = layer.capture(x, logits)
        ms_per_step, mode = timed(graph.replay), "hip-graph"

    # per-step spread (median and minimum over the same number of steps, one event pair per step) and the
    # device copy rate of this GPU, for reading the HBM fractions against something measured
    run_step = graph.replay if mode == "hip-graph" else step
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for a, b in evs:
        a.record()
        run_step()
        b.record()
    torch.cuda.synchronize()
    per_step = sorted(a.elapsed_time(b) for a, b in evs)
    step_median_ms, step_min_ms = per_step[len(per_step) // 2], per_step[0]
    cbuf = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    cdst = torch.empty_like(cbuf)
    copy_ms = time_events(lambda: cdst.copy_(cbuf), 10, torch)
    copy_gbs = 2.0 * cbuf.numel() / (copy_ms * 1e-3) / 1e9   # bytes read + bytes written
    del cbuf, cdst

    counts = np.diff(layer.expert_offsets.cpu().numpy())
    flops, min_bytes, R, active = algorithmic_work(shape, T, counts)
    tflops = flops / (ms_per_step * 1e-3) / 1e12
    gbs = min_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-call breakdown and the dominant kernel, events on the launch stream
    k, H, E = shape.top_k, shape.hidden, shape.n_experts
    rflags = (B.MOE_RENORM_TOPK if shape.renorm else 0) | (B.MOE_LOGITS_GIVEN if logits is not None else 0)
    it = max(5, min(steps, 50))
    br = {}
    br["route_topk"] = time_events(lambda: B.moe_route_topk(x, layer.w_router, layer.logits, T, H, E, k, rflags,
                                                            layer.topk_idx, layer.topk_w), it, torch)
    gather = layer.gathers(T)
    br["permute"] = time_events(lambda: B.moe_permute(x, layer.topk_idx, T, k, layer.shard,
                                                      None if gather else layer.x_perm,
                                                      layer.expert_offsets, layer.row_src, layer.slot_row,
                                                      layer.workspace), it, torch)
    if gather:   # the routed experts read their rows of x in place
        ffn = lambda fl: B.moe_expert_ffn_gather(x, layer.row_src, k, layer.expert_offsets, T * k, layer.ffn_shard,
                                                 layer.w_gate, layer.w_up, layer.w_down, layer.h_ws, layer.y_perm,
                                                 layer.ffn_ws, fl)
    else:
        ffn = lambda fl: B.moe_expert_ffn(layer.x_perm, layer.expert_offsets, T * k, layer.ffn_shard, layer.w_gate,
                                          layer.w_up, layer.w_down, layer.h_ws, layer.y_perm, layer.ffn_ws, fl)
    br["ffn_gateup_swiglu"] = time_events(lambda: ffn(B.MOE_FFN_SKIP_DOWN), it, torch)
    br["ffn_down"] = time_events(lambda: ffn(B.MOE_FFN_SKIP_GATEUP), it, torch)
    if layer.shared is not None:
        br["shared_expert_ffn"] = time_events(
            lambda: B.moe_expert_ffn(x, layer.sh_offsets, T, layer.shared_shard, *layer.shared, layer.h_sh,
                                     layer.y_shared, layer.ffn_ws_sh, 0), it, torch)
    br["combine"] = time_events(
        lambda: B.moe_combine(layer.y_perm, layer.slot_row, layer.topk_w, T, k, H,
                              layer.y_shared if layer.shared is not None else None,
                              x if layer.w_shared_gate is not None else None, layer.w_shared_gate, layer.y_out, 0),
        it, torch)

    # dominant kernel = GEMM1 (gate/up + SwiGLU): 2/3 of the routed FLOPs, 2/3 of the weight bytes
    g1_ms = br["ffn_gateup_swiglu"]
    I_s = shape.inter_slice
    g1_flops = 4.0 * R * H * I_s
    g1_bytes = 2.0 * active * H * I_s * 2 + R * H * 2 + R * I_s * 2
    intensity = g1_flops / g1_bytes
    decode = B.moe_debug_ffn_plan(T * k, layer.ffn_shard)[0]   # GEMM1 takes the weight-streaming kernel
    kname = ("moe::gw::grouped_walk_kernel<..., GATEUP> (GEMM1 + SwiGLU, weight streaming)" if decode
             else ("moe::gg::grouped_gemm_even_kernel<256, GATEUP> (GEMM1 + SwiGLU, 160-row blocks)"
                   if B.moe_debug_tile_rows(T * k, layer.ffn_shard) == 160
                   else "moe::gg::grouped_gemm_dlds_kernel<256, GATEUP> (GEMM1 + SwiGLU)"))
    if intensity > PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9):
        ach = g1_flops / (g1_ms * 1e-3) / 1e12
        roofline = {"kernel": kname, "bound": "mfma", "achieved": ach,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_BF16_TFLOPS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get(workload),
                    "ms": g1_ms, "flops_per_launch": g1_flops, "algorithmic_bytes_per_launch": g1_bytes}
    else:
        ach = g1_bytes / (g1_ms * 1e-3) / 1e9
        roofline = {"kernel": kname, "bound": "hbm", "achieved": ach,
                    "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get(workload),
                    "ms": g1_ms, "bytes_per_launch": g1_bytes}

    # the kernel's rate against both peaks (its own intensity decides which one `frac` is taken from)
    roofline["frac_of_mfma_peak"] = g1_flops / (g1_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS
    roofline["frac_of_hbm_peak"] = g1_bytes / (g1_ms * 1e-3) / 1e9 / PEAK_HBM_GBS
    roofline["flop_per_byte"] = intensity
    if 2.0 * active * H * I_s * 2 < 256e6:
        roofline["note"] = ("GEMM1's weights (%.0f MB) fit the 256 MB last-level cache and are replayed from one "
                            "buffer here: not an HBM measurement" % (2.0 * active * H * I_s * 2 / 1e6))

    return dict(shape=shape, T=T, desc=desc, li=li, layer=layer, x=x, logits=logits, ms_per_step=ms_per_step, mode=mode,
                eager_ms=eager_ms, step_median_ms=step_median_ms, step_min_ms=step_min_ms, copy_gbs=copy_gbs,
                flops=flops, min_bytes=min_bytes, R=R, active=active, tflops=tflops, gbs=gbs, br=br, gen_s=gen_s,
                roofline=roofline, k=k, H=H, E=E, I_s=I_s)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="mixtral_prefill", choices=sorted(WORKLOADS))
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 1 GiB device copies, to scale FETCH_SIZE / WRITE_SIZE counters under rocprofv3")
    ap.add_argument("--permuted-copy", action="store_true",
                    help="moe_permute writes x_perm and moe_expert_ffn reads it (default: the layer's own choice)")
    ap.add_argument("--gather-rows", action="store_true",
                    help="the FFN gathers its rows of x through row_src (default: the layer's own choice)")
    ap.add_argument("--no-overlap-shared", action="store_true",
                    help="run the shared expert after the routed experts instead of beside them on a second stream")
    ap.add_argument("--graph", choices=["auto", "on", "off"], default="auto",
                    help="replay the layer as one HIP graph (auto: when an eager step takes < 1 ms)")
    ap.add_argument("--cpu-sample-tokens", type=int, default=0, help="tokens the oracle is timed on (0 = auto)")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the other target shapes measured after the main workload")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU's shard: this build has no multi-GPU path; run with --gpus 1")

    import numpy as np
    import torch
    from paper_2508_19373_amd import binding as B
    from paper_2508_19373_amd import inputs as I
    from paper_2508_19373_amd.layer import ExpertShardLayer, bf16_tensor

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    B.lib()  # fail loudly when the HIP library is missing
    torch.cuda.set_device(0)

    if args.copy_calibration:  # a kernel of known traffic: reads 1 GiB, writes 1 GiB per launch
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    m = measure(args.workload, args.steps, args.warmup, args, torch, np, B, I, ExpertShardLayer, bf16_tensor)
    shape, T, desc, li, layer, x, logits = m["shape"], m["T"], m["desc"], m["li"], m["layer"], m["x"], m["logits"]
    ms_per_step, mode, eager_ms = m["ms_per_step"], m["mode"], m["eager_ms"]
    step_median_ms, step_min_ms, copy_gbs = m["step_median_ms"], m["step_min_ms"], m["copy_gbs"]
    flops, min_bytes, R, active, tflops, gbs = m["flops"], m["min_bytes"], m["R"], m["active"], m["tflops"], m["gbs"]
    br, gen_s, roofline, k, H, E, I_s = m["br"], m["gen_s"], m["roofline"], m["k"], m["H"], m["E"], m["I_s"]

    # ---- CPU baseline: the oracle as it stands on a bounded token sample
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moe_oracle as O
        n = args.cpu_sample_tokens or min(T, 4096)
        sel = np.linspace(0, T - 1, n).astype(np.int64)
        lg = layer.logits[:T].cpu().numpy()[sel]
        shared = (li.ws_gate, li.ws_up, li.ws_down) if li.ws_gate is not None else None
        t0 = time.perf_counter()
        ref = O.expert_layer(li.x[sel], lg, k, shape.renorm, shape.n_local_experts, shape.expert_offset, li.w_gate,
                             li.w_up, li.w_down, shared=shared,
                             w_shared_gate=li.w_shared_gate if shared else None)
        cpu_s = time.perf_counter() - t0
        idx_s, _, _ = O.route_topk(lg, k, shape.renorm)
        cnt_s = [int(((idx_s >= shape.expert_offset + e) & (idx_s < shape.expert_offset + e + 1)).sum())
                 for e in range(shape.n_local_experts)]
        f_s, _, _, _ = algorithmic_work(shape, n, cnt_s)
        got = layer.y_out[:T].float().cpu().numpy()[sel].astype(np.float64)
        rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30))
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        cpu = {"value": f_s / cpu_s / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
               "sample": "%d of %d tokens (evenly spaced), full weights, fp64 numpy; %.1f s" % (n, T, cpu_s),
               "gpu_vs_oracle_rel_l2_on_sample": rel}

    out = {
        "metric": "moe_expert_layer_bf16_tflops", "value": tflops, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "us_per_layer": ms_per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": desc, "tokens": T, "routed_rows": R, "active_local_experts": active,
                   "hidden": H, "n_experts": E, "top_k": k, "inter_slice": I_s,
                   "n_local_experts": shape.n_local_experts, "expert_offset": shape.expert_offset, "seed": args.seed},
        "pct_mfma_peak": 100.0 * tflops / PEAK_BF16_TFLOPS, "min_bytes_gbs": gbs,
        "pct_hbm_peak": 100.0 * gbs / PEAK_HBM_GBS, "flops_per_layer": flops, "min_bytes_per_layer": min_bytes,
        "launch_mode": mode, "eager_ms_per_step": eager_ms, "step_ms_median": step_median_ms,
        "step_ms_min": step_min_ms, "device_copy_gbs": copy_gbs, "breakdown_ms": br, "input_gen_s": gen_s, "roofline": roofline, "cpu_baseline": cpu,
    }
    # ---- the other target shapes in the same process, so that one run of the default command covers
    # every shape the targets are stated for
    if not args.no_also:
        del m, layer, x, logits, li
        torch.cuda.empty_cache()
        also = {}
        for w in ALSO_WORKLOADS:
            if w == args.workload:
                continue
            # (their own step counts: short runs of these small layers are dominated by the clock settling)
            try:
                a = measure(w, 50, 30, args, torch, np, B, I, ExpertShardLayer, bf16_tensor)
            except Exception as e:  # the headline line is printed whatever happens to an extra workload
                also[w] = {"error": "%s: %s" % (type(e).__name__, e)}
                continue
            r = a["roofline"]
            also[w] = {"workload": a["desc"], "us_per_layer": a["ms_per_step"] * 1e3, "launch_mode": a["mode"],
                       "tflops": a["tflops"], "pct_mfma_peak": 100.0 * a["tflops"] / PEAK_BF16_TFLOPS,
                       "min_bytes_gbs": a["gbs"], "pct_hbm_peak": 100.0 * a["gbs"] / PEAK_HBM_GBS,
                       "bound": r["bound"], "frac": r["frac"], "traffic": r["traffic"], "kernel": r["kernel"],
                       "kernel_ms": r["ms"],
                       "breakdown_ms": a["br"]}
            del a
            torch.cuda.empty_cache()
        out["also"] = also
    print(json.dumps(out))


if __name__ == "__main__":
    main()
