"""Seeded synthetic inputs for the MoE Expert-module shard path.

This module holds no arithmetic of the method itself (no routing, no GEMM, no
softmax): it only draws random tensors of the shapes the paper's workloads have
(model table in the evaluation section: Mixtral-8x7B hidden 4096 / 8 experts /
intermediate 14336, Qwen1.5-MoE-A2.7B hidden 2048 / 60 experts / intermediate
1408, Qwen2-57B-A14B hidden 3584 / 64 experts / intermediate 2560) and encodes
them as bf16.  What that table leaves open (top-k, shared-expert size, gate
renormalisation) follows the published model configurations: top-2 with
renormalisation for Mixtral, top-4 plus a 5632-wide shared expert for
Qwen1.5-MoE, top-8 plus a 20480-wide shared expert for Qwen2-57B-A14B.  Both the HIP path's tests and the CPU oracle's
tests take their inputs from here; neither side's code lives here.

bf16 tensors are carried as ``numpy.uint16`` bit patterns so that numpy (which
has no bf16 type) and torch (``tensor.view(torch.bfloat16)``) see the same bits.

Every tensor is a pure function of ``(seed, tensor id, sub-index)`` through
numpy's counter-based Philox generator, so a shard can draw exactly its own
slice of a weight matrix without materialising the rest.  Expert weights are
drawn in ``N_INTER_BLOCKS`` blocks along the intermediate dimension; a tensor
parallel shard of degree ``E_t`` (a power of two up to 8, as in the paper's
search-space section) owns a contiguous run of those blocks.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np

# tensor ids (fixed so that a seed names one data set)
TID_X, TID_WR, TID_WG, TID_WU, TID_WD, TID_SHARED, TID_WS, TID_GUMBEL = range(8)
N_INTER_BLOCKS = 8  # max tensor-parallel degree the generator can slice for

_POOL_THREADS = 8


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact bf16 (uint16 bits) -> fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed: int, tid: int, *sub: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([int(seed), int(tid), *map(int, sub)])))


@dataclass(frozen=True)
class MoEShape:
    """One workload: the full (unsharded) layer plus which shard of it is run."""
    name: str
    hidden: int            # H
    n_experts: int         # E
    top_k: int             # k
    inter: int             # I (expert intermediate size, full)
    renorm: bool           # renormalise the k selected gate weights to sum 1
    inter_shared: int = 0  # shared-expert intermediate size, 0 = no shared expert
    router: str = "normal"  # "normal" N(0,0.02) | "uniform" U(-a,a) same variance | "zipf" logits given
    tp_degree: int = 1     # E_t
    tp_rank: int = 0
    ep_degree: int = 1     # E_e
    ep_rank: int = 0

    @property
    def n_local_experts(self) -> int:
        return self.n_experts // self.ep_degree

    @property
    def expert_offset(self) -> int:
        return self.ep_rank * self.n_local_experts

    @property
    def inter_slice(self) -> int:
        return self.inter // self.tp_degree

    @property
    def inter_shared_slice(self) -> int:
        return self.inter_shared // self.tp_degree

    def shard(self, tp_degree=1, tp_rank=0, ep_degree=1, ep_rank=0) -> "MoEShape":
        return replace(self, tp_degree=tp_degree, tp_rank=tp_rank, ep_degree=ep_degree, ep_rank=ep_rank)


# The five workloads of the benchmark plan.  Token counts are given separately.
TINY = MoEShape("tiny", 512, 8, 2, 1024, True)
MIXTRAL = MoEShape("mixtral-8x7b", 4096, 8, 2, 14336, True, router="uniform")
MIXTRAL_TP4 = replace(MIXTRAL, name="mixtral-8x7b-tp4", tp_degree=4, tp_rank=0)
MIXTRAL_EP4_HOT = replace(MIXTRAL, name="mixtral-8x7b-ep4-hot", router="zipf", ep_degree=4, ep_rank=0)
MIXTRAL_EP4_COLD = replace(MIXTRAL, name="mixtral-8x7b-ep4-cold", router="zipf", ep_degree=4, ep_rank=3)
QWEN = MoEShape("qwen1.5-moe-a2.7b", 2048, 60, 4, 1408, False, inter_shared=5632)
QWEN2_57B = MoEShape("qwen2-57b-a14b", 3584, 64, 8, 2560, False, inter_shared=20480)

WORKLOADS: Dict[str, Tuple[MoEShape, Tuple[int, ...]]] = {
    "tiny": (TINY, (64,)),
    "mixtral": (MIXTRAL, (16, 4096)),
    "mixtral_tp4": (MIXTRAL_TP4, (64, 8192)),
    "mixtral_ep4_hot": (MIXTRAL_EP4_HOT, (8192,)),
    "mixtral_ep4_cold": (MIXTRAL_EP4_COLD, (8192,)),
    "qwen": (QWEN, (32, 4096)),
    "qwen2_57b": (QWEN2_57B, (32, 4096)),
}

ZIPF_S = 1.2


def make_x(seed: int, T: int, H: int) -> np.ndarray:
    """Token activations x ~ N(0,1), bf16 bits [T,H].  Row t depends only on (seed, t)
    block-wise, so a prefix of a larger batch equals the smaller batch."""
    return f32_to_bf16_bits(_rng(seed, TID_X).standard_normal((T, H), dtype=np.float32))


def make_router_weight(seed: int, shape: MoEShape) -> Optional[np.ndarray]:
    """Router weight W_r [H,E] fp32 (row-major).  None when the workload supplies logits."""
    H, E = shape.hidden, shape.n_experts
    g = _rng(seed, TID_WR)
    if shape.router == "normal":
        return (0.02 * g.standard_normal((H, E), dtype=np.float32)).astype(np.float32)
    if shape.router == "uniform":
        a = 0.02 * math.sqrt(3.0)  # same variance as N(0, 0.02)
        return g.uniform(-a, a, size=(H, E)).astype(np.float32)
    return None


def zipf_popularity(E: int, s: float = ZIPF_S) -> np.ndarray:
    p = 1.0 / np.arange(1, E + 1, dtype=np.float64) ** s
    return p / p.sum()


def make_zipf_logits(seed: int, T: int, E: int, s: float = ZIPF_S) -> np.ndarray:
    """Router logits ln p_e + Gumbel noise (fp32 [T,E]) so that the first choice of
    every token is expert e with probability p_e ~ (e+1)^-s exactly."""
    u = _rng(seed, TID_GUMBEL).random((T, E), dtype=np.float64)
    u = np.clip(u, 1e-300, 1.0 - 1e-16)
    gumbel = -np.log(-np.log(u))
    return (np.log(zipf_popularity(E, s))[None, :] + gumbel).astype(np.float32)


def _weight_block(seed: int, tid: int, expert: int, block: int, rows: int, cols: int) -> np.ndarray:
    w = _rng(seed, tid, expert, block).standard_normal((rows, cols), dtype=np.float32)
    w *= np.float32(0.02)
    return f32_to_bf16_bits(w)


def _blocks_of_shard(shape: MoEShape) -> range:
    per = N_INTER_BLOCKS // shape.tp_degree
    return range(shape.tp_rank * per, (shape.tp_rank + 1) * per)


def make_expert_weights(seed: int, shape: MoEShape, *, shared: bool = False):
    """Weights of the shard's local experts, bf16 bits:
    gate, up  [E_loc, I_s, H]   (row i = output feature i, H contiguous)
    down      [E_loc, H, I_s]   (row n = output feature n, I_s contiguous)
    ``shared=True`` draws the single shared expert instead (E_loc = 1, size inter_shared).
    Each is N(0, 0.02) rounded to bf16.  The tensor-parallel slice is rows
    [p*I_s, (p+1)*I_s) of gate/up and the same columns of down.
    """
    if shape.tp_degree not in (1, 2, 4, 8):
        raise ValueError("tp_degree must be 1, 2, 4 or 8")
    H = shape.hidden
    if shared:
        I_full, experts, tids = shape.inter_shared, [0], (TID_SHARED, TID_SHARED, TID_SHARED)
        kind_base = (0, 1, 2)
    else:
        I_full = shape.inter
        experts = list(range(shape.expert_offset, shape.expert_offset + shape.n_local_experts))
        tids, kind_base = (TID_WG, TID_WU, TID_WD), (0, 0, 0)
    if I_full % N_INTER_BLOCKS:
        raise ValueError("intermediate size must be a multiple of %d" % N_INTER_BLOCKS)
    bi = I_full // N_INTER_BLOCKS
    blocks = list(_blocks_of_shard(shape))
    I_s = bi * len(blocks)
    n = len(experts)
    wg = np.empty((n, I_s, H), np.uint16)
    wu = np.empty((n, I_s, H), np.uint16)
    wd = np.empty((n, H, I_s), np.uint16)

    def job(args):
        which, le, e, lb, b = args
        if which == 0:
            wg[le, lb * bi:(lb + 1) * bi, :] = _weight_block(seed, tids[0], e * 4 + kind_base[0], b, bi, H)
        elif which == 1:
            wu[le, lb * bi:(lb + 1) * bi, :] = _weight_block(seed, tids[1], e * 4 + kind_base[1], b, bi, H)
        else:
            wd[le, :, lb * bi:(lb + 1) * bi] = _weight_block(seed, tids[2], e * 4 + kind_base[2], b, H, bi)

    jobs = [(w, le, e, lb, b) for le, e in enumerate(experts) for lb, b in enumerate(blocks) for w in range(3)]
    with ThreadPoolExecutor(_POOL_THREADS) as pool:
        list(pool.map(job, jobs))
    return wg, wu, wd


def make_shared_gate_weight(seed: int, H: int) -> np.ndarray:
    """w_s [H] fp32 ~ N(0,0.02), rounded so every value is bf16-representable."""
    w = (0.02 * _rng(seed, TID_WS).standard_normal(H, dtype=np.float32)).astype(np.float32)
    return bf16_bits_to_f32(f32_to_bf16_bits(w))


@dataclass
class LayerInputs:
    shape: MoEShape
    T: int
    seed: int
    x: np.ndarray                     # [T,H] bf16 bits
    w_router: Optional[np.ndarray]    # [H,E] fp32 or None
    logits: Optional[np.ndarray]      # [T,E] fp32 when the workload supplies logits
    w_gate: np.ndarray                # [E_loc,I_s,H] bf16 bits
    w_up: np.ndarray
    w_down: np.ndarray                # [E_loc,H,I_s] bf16 bits
    ws_gate: Optional[np.ndarray] = None   # shared expert [1,I_sh_s,H]
    ws_up: Optional[np.ndarray] = None
    ws_down: Optional[np.ndarray] = None   # [1,H,I_sh_s]
    w_shared_gate: Optional[np.ndarray] = None  # [H] fp32


def make_layer_inputs(shape: MoEShape, T: int, seed: int = 0, *, weights: bool = True) -> LayerInputs:
    """All inputs of one Expert-module call on one shard."""
    x = make_x(seed, T, shape.hidden)
    w_r = make_router_weight(seed, shape)
    logits = make_zipf_logits(seed, T, shape.n_experts) if shape.router == "zipf" else None
    if weights:
        wg, wu, wd = make_expert_weights(seed, shape)
    else:
        wg = wu = wd = None
    out = LayerInputs(shape, T, seed, x, w_r, logits, wg, wu, wd)
    if shape.inter_shared:
        if weights:
            out.ws_gate, out.ws_up, out.ws_down = make_expert_weights(seed, shape, shared=True)
        out.w_shared_gate = make_shared_gate_weight(seed, shape.hidden)
    return out
