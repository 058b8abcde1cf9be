"""Optimal hybrid parallel strategy search (paper, "Optimal Hybrid Parallel Strategies Search" and
"The Dynamic Parallelism Transition Strategy").  CPU only.

The paper states the problem as an integer linear program over one-hot vectors S_k (Attention
strategy), E_i (Expert strategy in prefill) and E_j (Expert strategy in decoding):

    min  N_layer * { (T_a[k] + T_e^pre[i] + T_C^pre[k,i]) + S_out * (T_a^dec[k] + T_e^dec[j] + T_C^dec[k,j]) } + C[i,j]

subject to the memory bound (M_KV + A_d*M_attn + E_d*M_exp)/N + 2*M_act < M_gpu, N = A_t*A_d =
E_d*E_t*E_e, and the divisibility rules (TP degrees powers of two that divide the head counts /
the expert intermediate size, EP degree dividing the expert count).  DP is excluded for the Expert
module (E_d = 1) and so is the DP+EP+TP triple.  The space is tiny (K_a <= 4, K_e <= 4 on 8
devices), so instead of an ILP solver the search enumerates it and is exact by construction.

Cost inputs:
  T_e    the Expert-module latency table this repository measures on MI355X
         (profiles/expert_latency_table_mi355x.csv), interpolated in log(tokens);
  T_deq  the measured V_dequant -> T_dequant dictionary (profiles/int4_dequant_table_mi355x.csv);
  T_a, T_C, T_upload, T_reshard  analytic placeholders (roofline attention, alpha-beta collectives
         on an 8-GPU xGMI full mesh, PCIe upload): they are not measured here -- one GPU -- and are
         stated as such; `Hardware` holds every constant.
The switching cost follows the paper's formula per layer, C_ij = min{T_reshard, max{0, T_upload +
T_dequant - T_prefill_layer}}, and is charged once per layer (every layer's expert weights move).
"""
from __future__ import annotations

import csv
import math
import os
from dataclasses import dataclass
from itertools import product
from typing import Dict, List, Optional, Sequence, Tuple

from . import dequant_table as D

_PROFILES = os.path.join(os.path.dirname(os.path.abspath(__file__)), "..", "profiles")


@dataclass(frozen=True)
class ModelConfig:
    """What the search needs to know of a model (evaluation-section model table; head counts and
    layer counts from the published configurations)."""
    name: str
    n_layers: int
    hidden: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    n_experts: int
    top_k: int
    inter: int
    inter_shared: int = 0

    @property
    def expert_params_per_layer(self) -> int:
        return 3 * self.hidden * (self.n_experts * self.inter + self.inter_shared)

    @property
    def attn_params_per_layer(self) -> int:
        q = self.n_heads * self.head_dim
        kv = self.n_kv_heads * self.head_dim
        return self.hidden * (2 * q + 2 * kv)


MIXTRAL_8X7B = ModelConfig("mixtral-8x7b", 32, 4096, 32, 8, 128, 8, 2, 14336)
QWEN15_MOE = ModelConfig("qwen1.5-moe-a2.7b", 24, 2048, 16, 16, 128, 60, 4, 1408, 5632)
QWEN2_57B = ModelConfig("qwen2-57b-a14b", 28, 3584, 28, 4, 128, 64, 8, 2560, 20480)
MODELS = {m.name: m for m in (MIXTRAL_8X7B, QWEN15_MOE, QWEN2_57B)}


@dataclass(frozen=True)
class Hardware:
    """Constants of the analytic placeholders (an 8 x MI355X node)."""
    n_devices: int = 8
    mem_bytes: float = 288e9 * 0.9          # usable HBM per GPU
    peak_flops: float = 2.5e15 * 0.5        # attention GEMMs at half of the bf16 MFMA peak
    hbm_bw: float = 8e12 * 0.7              # streaming kernels at 70 % of the HBM peak
    link_bw: float = 153.6e9 * 0.8          # one xGMI link, per direction, at 80 %
    coll_latency: float = 15e-6             # per collective
    pcie_bw: float = 64e9 * 0.8             # host-to-device upload (PCIe 5 x16)
    act_factor: float = 4.0                 # M_act = act_factor * b * s * hidden * 2 bytes


@dataclass(frozen=True)
class Scenario:
    batch: int      # B, sequences in flight on the node
    s_in: int       # prompt tokens per sequence
    s_out: int      # generated tokens per sequence


def _pow2_upto(n: int) -> List[int]:
    return [1 << i for i in range(n.bit_length()) if (1 << i) <= n]


def attention_strategies(m: ModelConfig, n_devices: int) -> List[Tuple[int, int]]:
    """(A_t, A_d): A_t * A_d = N, A_t a power of two dividing the query and KV head counts."""
    return [(t, n_devices // t) for t in _pow2_upto(n_devices)
            if n_devices % t == 0 and m.n_heads % t == 0 and m.n_kv_heads % t == 0]


def expert_strategies(m: ModelConfig, n_devices: int) -> List[Tuple[int, int]]:
    """(E_t, E_e): E_t * E_e = N (no DP for experts), E_t a power of two dividing the expert
    intermediate size (and the shared expert's), E_e dividing the expert count."""
    out = []
    for t in _pow2_upto(n_devices):
        e = n_devices // t
        if n_devices % t or m.inter % t or m.inter_shared % t or m.n_experts % e:
            continue
        out.append((t, e))
    return out


def memory_ok(m: ModelConfig, hw: Hardware, sc: Scenario, attn: Tuple[int, int], e_d: int = 1) -> bool:
    """(M_KV + A_d*M_attn + E_d*M_exp)/N + 2*M_act < M_gpu, bf16 everywhere."""
    a_t, a_d = attn
    m_kv = sc.batch * (sc.s_in + sc.s_out) * m.n_layers * 2 * m.n_kv_heads * m.head_dim * 2.0
    m_attn = m.n_layers * m.attn_params_per_layer * 2.0
    m_exp = m.n_layers * m.expert_params_per_layer * 2.0
    b = sc.batch / a_d
    m_act = hw.act_factor * b * sc.s_in * m.hidden * 2.0
    return (m_kv + a_d * m_attn + e_d * m_exp) / hw.n_devices + 2.0 * m_act < hw.mem_bytes


# --------------------------------------------------------------------------- cost vectors
class ExpertLatencyTable:
    """T_e from the measured table: microseconds per layer of one shard, by (model, E_t, E_e),
    interpolated linearly in (log tokens, log latency)."""

    def __init__(self, path: Optional[str] = None):
        path = path or os.path.join(_PROFILES, "expert_latency_table_mi355x.csv")
        self.curves: Dict[Tuple[str, int, int], List[Tuple[float, float]]] = {}
        with open(path) as f:
            for r in csv.DictReader(f):
                if r.get("routing", "balanced") != "balanced":
                    continue  # the search's T_e is the balanced-routing curve of each shard
                key = (r["model"], int(r["tp"]), int(r["ep"]))
                self.curves.setdefault(key, []).append((math.log(float(r["tokens"])), math.log(float(r["us_per_layer"]))))
        for c in self.curves.values():
            c.sort()

    def seconds(self, model: str, e_t: int, e_e: int, tokens: float) -> float:
        c = self.curves[(model, e_t, e_e)]
        x = math.log(max(tokens, 1.0))
        if x <= c[0][0]:
            return math.exp(c[0][1]) * 1e-6
        for (x0, y0), (x1, y1) in zip(c, c[1:]):
            if x <= x1:
                return math.exp(y0 + (y1 - y0) * (x - x0) / (x1 - x0)) * 1e-6
        (x0, y0), (x1, y1) = c[-2], c[-1]   # beyond the table: the last log-log slope
        return math.exp(y1 + (y1 - y0) * (x - x1) / (x1 - x0)) * 1e-6


def attention_seconds(m: ModelConfig, hw: Hardware, attn: Tuple[int, int], seqs: float, q_len: int, ctx: int) -> float:
    """Placeholder T_a of one layer on one device: roofline of the projections and the score /
    value products for `seqs / A_d` sequences, heads split A_t ways."""
    a_t, a_d = attn
    toks = seqs / a_d * q_len
    flops = 2.0 * toks * m.attn_params_per_layer / a_t + 4.0 * toks * ctx * m.n_heads * m.head_dim / a_t * (0.5 if q_len > 1 else 1.0)
    bytes_ = m.attn_params_per_layer * 2.0 / a_t + seqs / a_d * ctx * 2 * m.n_kv_heads * m.head_dim * 2.0 / a_t
    return max(flops / hw.peak_flops, bytes_ / hw.hbm_bw)


def _all_reduce(hw: Hardware, bytes_: float, group: int) -> float:
    # direct reduce-scatter + all-gather on a full mesh: every peer link carries bytes/group, twice
    return 0.0 if group <= 1 else hw.coll_latency + 2.0 * (bytes_ / group) / hw.link_bw


def _all_gather(hw: Hardware, bytes_out: float, group: int) -> float:
    return 0.0 if group <= 1 else hw.coll_latency + (bytes_out / group) / hw.link_bw


def _all_to_all(hw: Hardware, bytes_per_device: float, group: int) -> float:
    return 0.0 if group <= 1 else hw.coll_latency + (bytes_per_device / group) / hw.link_bw


def comm_seconds(m: ModelConfig, hw: Hardware, attn: Tuple[int, int], exp: Tuple[int, int], tokens: float) -> float:
    """Placeholder T_C of one layer for the pair (Attention strategy, Expert strategy); `tokens`
    is the node-wide token count of the step.  Attention TP: all-reduce of its output inside the
    TP group.  Expert module: tokens of the A_d data-parallel groups are gathered to every device
    of the TP dimension; across the EP dimension rows travel by all-to-all (dispatch and combine)
    when attention is data parallel, else only the outputs are reduced."""
    a_t, a_d = attn
    e_t, e_e = exp
    row = m.hidden * 2.0
    t = _all_reduce(hw, tokens / a_d * row, a_t)
    if e_e > 1:
        if a_d > 1:   # rows leave their DP group for the expert's device and come back
            t += 2.0 * _all_to_all(hw, tokens / a_d * m.top_k * row, e_e)
        else:         # every device already holds all tokens: reduce the EP partial outputs
            t += _all_reduce(hw, tokens * row, e_e)
    if e_t > 1:
        gather = tokens * row if a_d > 1 else 0.0     # all tokens to every TP rank
        t += _all_gather(hw, gather, e_t) + _all_reduce(hw, tokens * row / max(e_e, 1), e_t)
    return t


def switching_seconds(m: ModelConfig, hw: Hardware, exp_i: Tuple[int, int], exp_j: Tuple[int, int],
                      prefill_layer_s: float, dequant_rows) -> float:
    """Whole-model switching cost from Expert strategy i (prefill) to j (decoding):
    N_layer * min{T_reshard, max{0, T_upload + T_dequant - T_prefill_layer}}."""
    if exp_i == exp_j:
        return 0.0
    v = m.expert_params_per_layer // hw.n_devices          # V_dequant: one device's new shard of a layer
    t_upload = v * D.BYTES_PER_WEIGHT_IN / hw.pcie_bw
    t_dequant = D.lookup(dequant_rows, v) * 1e-6
    # reshard by collectives: the new shard arrives over the mesh (all-to-all of bf16 weights)
    t_reshard = hw.coll_latency + (v * 2.0 / hw.n_devices) / hw.link_bw * (hw.n_devices - 1)
    return m.n_layers * min(t_reshard, max(0.0, t_upload + t_dequant - prefill_layer_s))


# --------------------------------------------------------------------------- the search
@dataclass
class Choice:
    attention: Tuple[int, int]
    expert_prefill: Tuple[int, int]
    expert_decode: Tuple[int, int]
    total_s: float
    prefill_s: float
    decode_s: float
    switch_s: float


def cost_tensors(m: ModelConfig, hw: Hardware, sc: Scenario, t_e: ExpertLatencyTable, dequant_rows):
    """The ILP's inputs: strategy lists K_a, K_e, per-layer cost arrays pre[k][i], dec[k][j] (T_a +
    T_e + T_C) and the switching matrix C[k][i][j] (it depends on k through the prefill time)."""
    ka = [a for a in attention_strategies(m, hw.n_devices) if memory_ok(m, hw, sc, a)]
    ke = expert_strategies(m, hw.n_devices)
    pre_tokens, dec_tokens = sc.batch * sc.s_in, sc.batch
    ctx_dec = sc.s_in + sc.s_out // 2
    pre = [[attention_seconds(m, hw, a, sc.batch, sc.s_in, sc.s_in) + t_e.seconds(m.name, e[0], e[1], pre_tokens)
            + comm_seconds(m, hw, a, e, pre_tokens) for e in ke] for a in ka]
    dec = [[attention_seconds(m, hw, a, sc.batch, 1, ctx_dec) + t_e.seconds(m.name, e[0], e[1], dec_tokens)
            + comm_seconds(m, hw, a, e, dec_tokens) for e in ke] for a in ka]
    sw = [[[switching_seconds(m, hw, ei, ej, pre[k][i], dequant_rows) for ej in ke] for i, ei in enumerate(ke)]
          for k in range(len(ka))]
    return ka, ke, pre, dec, sw


def exact_search(n_layers: int, s_out: int, pre: Sequence[Sequence[float]], dec: Sequence[Sequence[float]],
                 sw: Sequence[Sequence[Sequence[float]]]) -> Tuple[Tuple[int, int, int], float]:
    """argmin over (k, i, j) of N_layer * (pre[k][i] + S_out * dec[k][j]) + C[k][i][j]; ties go to
    the first triple in lexicographic order."""
    best, arg = math.inf, None
    for k, i, j in product(range(len(pre)), range(len(pre[0]) if pre else 0), range(len(dec[0]) if dec else 0)):
        v = n_layers * (pre[k][i] + s_out * dec[k][j]) + sw[k][i][j]
        if v < best:
            best, arg = v, (k, i, j)
    return arg, best


def search(m: ModelConfig, sc: Scenario, hw: Hardware = Hardware(), t_e: Optional[ExpertLatencyTable] = None,
           dequant_rows=None) -> Choice:
    t_e = t_e or ExpertLatencyTable()
    dequant_rows = dequant_rows or D.load(os.path.join(_PROFILES, "int4_dequant_table_mi355x.csv"))
    ka, ke, pre, dec, sw = cost_tensors(m, hw, sc, t_e, dequant_rows)
    if not ka or not ke:
        raise ValueError("no feasible strategy: the memory bound excludes every Attention strategy")
    (k, i, j), total = exact_search(m.n_layers, sc.s_out, pre, dec, sw)
    return Choice(ka[k], ke[i], ke[j], total, m.n_layers * pre[k][i], m.n_layers * sc.s_out * dec[k][j], sw[k][i][j])


def tp_baseline(m: ModelConfig, sc: Scenario, hw: Hardware = Hardware(), t_e: Optional[ExpertLatencyTable] = None,
                dequant_rows=None) -> float:
    """Latency of the paper's comparison point under the same cost model: TP everywhere."""
    t_e = t_e or ExpertLatencyTable()
    dequant_rows = dequant_rows or D.load(os.path.join(_PROFILES, "int4_dequant_table_mi355x.csv"))
    ka, ke, pre, dec, sw = cost_tensors(m, hw, sc, t_e, dequant_rows)
    k = max(range(len(ka)), key=lambda q: ka[q][0])
    i = max(range(len(ke)), key=lambda q: ke[q][0])
    return m.n_layers * (pre[k][i] + sc.s_out * dec[k][i])


def main():
    # the paper's four scenarios (context, generation), on one 8-GPU node
    scenarios = [(256, 64), (256, 2048), (4096, 64), (4096, 2048)]
    print("%-20s %-12s %-9s %-9s %-9s %10s %10s %8s" % ("model", "scenario", "attention", "exp/pre", "exp/dec",
                                                      "total ms", "TP ms", "speedup"))
    for m in MODELS.values():
        for s_in, s_out in scenarios:
            sc = Scenario(batch=8, s_in=s_in, s_out=s_out)
            c = search(m, sc)
            base = tp_baseline(m, sc)
            fmt = lambda s, names: "%s%dx%s%d" % (names[0], s[0], names[1], s[1])
            print("%-20s %-12s %-9s %-9s %-9s %10.2f %10.2f %8.3f" % (
                m.name, "%d/%d" % (s_in, s_out), fmt(c.attention, ("TP", "DP")), fmt(c.expert_prefill, ("TP", "EP")),
                fmt(c.expert_decode, ("TP", "EP")), c.total_s * 1e3, base * 1e3, base / c.total_s))


if __name__ == "__main__":
    main()
