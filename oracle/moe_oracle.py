"""CPU oracle for the MoE Expert-module forward pass on one shard.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path is
checked against.  It may be imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path.  It shares no code with
the HIP library and does not import it.

What it computes (paper, "MoE Model Architectures": an Expert module is a gating
network with Top-K selection that dispatches each token to its most relevant expert
networks; some models add always-active shared experts; "Tensor Parallelism"
partitions the expert weights, "Expert Parallelism" distributes whole experts; the
ILP constraints require the expert count to be divisible by the EP degree and the
expert intermediate size by the TP degree).  The paper states the layer in words
only; the concrete definition (softmax over all experts then top-k, optional
renormalisation, SwiGLU experts without biases, sigmoid-gated shared expert) is the
reading documented in the design notes of this repository.

Everything is evaluated in float64 from exactly-converted inputs, with no blocking,
fusion or intermediate rounding.  numpy's matmul serves as the dot-product step.

Pins (tests/test_oracle_pins.py): brute-force dense evaluation of every expert with
masked gate weights; TP shard partial sums add up to the unsharded output; EP shard
outputs add up to the full layer; tie-break and softmax special cases; library
stable sort for the permutation; E=1,k=1 reduces to a three-matmul SwiGLU MLP;
token-permutation equivariance; identical experts with k=E.  The paper prints no
worked numeric example for this path, so beyond those pins parity is unpinned.
"""
from __future__ import annotations

import numpy as np


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact bf16 (uint16 bit patterns) -> float64."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------- routing
def router_logits(x_bits: np.ndarray, w_router: np.ndarray) -> np.ndarray:
    """Gating-network logits L[t,e] = sum_h x[t,h] W_r[h,e], fp64 sum, one rounding to fp32."""
    x = bf16_to_f64(x_bits)
    w = np.asarray(w_router, dtype=np.float32).astype(np.float64)
    return (x @ w).astype(np.float32)


def route_topk(logits: np.ndarray, k: int, renorm: bool):
    """Top-K selection of the gating network.

    Experts are ordered by (logit descending, expert index ascending); the first k
    are selected, in that order.  Gate weight = softmax over ALL experts evaluated at
    the selected ones; with ``renorm`` the k weights are divided by their sum.
    Returns (idx int32 [T,k], w float32 [T,k], w64 float64 [T,k]).
    """
    L32 = np.asarray(logits, dtype=np.float32)
    if not np.all(np.isfinite(L32)):
        raise ValueError("non-finite logits are outside the contract")
    T, E = L32.shape
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    L = L32.astype(np.float64)
    idx = np.empty((T, k), np.int32)
    for t in range(T):
        # -0.0 == +0.0 compares equal, so the expert index breaks that tie too
        order = sorted(range(E), key=lambda e: (-L[t, e], e))
        idx[t, :] = order[:k]
    m = L.max(axis=1, keepdims=True)
    p = np.exp(L - m)
    p /= p.sum(axis=1, keepdims=True)
    w = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return idx, w.astype(np.float32), w


# --------------------------------------------------------------------------- permutation
def permute(x_bits: np.ndarray, idx: np.ndarray, n_local_experts: int, expert_offset: int):
    """Stable counting sort of the local (token, slot) assignments by expert.

    Assignment a = t*k + j goes to expert idx[t,j]; it is local iff
    expert_offset <= idx[t,j] < expert_offset + n_local_experts (EP holds a
    contiguous subset of experts).  Rows of one expert keep increasing a.
    Returns expert_offsets [E_loc+1], row_src [R], slot_row [T*k], x_perm [R,H] (bits).
    """
    T, k = idx.shape
    flat = np.asarray(idx, dtype=np.int64).reshape(-1)
    counts = np.zeros(n_local_experts, np.int64)
    for a in range(T * k):
        e = flat[a] - expert_offset
        if 0 <= e < n_local_experts:
            counts[e] += 1
    expert_offsets = np.zeros(n_local_experts + 1, np.int32)
    expert_offsets[1:] = np.cumsum(counts)
    R = int(expert_offsets[-1])
    fill = expert_offsets[:-1].astype(np.int64).copy()
    row_src = np.empty(R, np.int32)
    slot_row = np.full(T * k, -1, np.int32)
    for a in range(T * k):
        e = flat[a] - expert_offset
        if 0 <= e < n_local_experts:
            r = fill[e]
            fill[e] += 1
            row_src[r] = a
            slot_row[a] = r
    x_perm = np.asarray(x_bits)[row_src // k] if R else np.zeros((0, x_bits.shape[1]), x_bits.dtype)
    return expert_offsets, row_src, slot_row, x_perm


# --------------------------------------------------------------------------- experts
def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def expert_ffn(x_perm_bits: np.ndarray, expert_offsets: np.ndarray,
               w_gate_bits: np.ndarray, w_up_bits: np.ndarray, w_down_bits: np.ndarray) -> np.ndarray:
    """SwiGLU expert networks on the permuted rows, float64, no intermediate rounding.

    For the rows r of local expert e:  g = x_r Wg_e^T, u = x_r Wu_e^T,
    h = silu(g) * u,  y_r = h Wd_e^T.  Weights are the shard's slice
    (gate/up [E_loc,I_s,H], down [E_loc,H,I_s]); with I_s < I the result is the
    tensor-parallel partial sum (no all-reduce).
    Returns y_perm [R,H] float64.
    """
    R = int(expert_offsets[-1])
    H = w_down_bits.shape[1]
    y = np.zeros((R, H), np.float64)
    for e in range(len(expert_offsets) - 1):
        lo, hi = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if hi == lo:
            continue
        xe = bf16_to_f64(x_perm_bits[lo:hi])
        g = xe @ bf16_to_f64(w_gate_bits[e]).T
        u = xe @ bf16_to_f64(w_up_bits[e]).T
        h = silu(g) * u
        y[lo:hi] = h @ bf16_to_f64(w_down_bits[e]).T
    return y


def shared_gate(x_bits: np.ndarray, w_shared_gate: np.ndarray) -> np.ndarray:
    """sigmoid(x . w_s) per token, float64 [T]."""
    z = bf16_to_f64(x_bits) @ np.asarray(w_shared_gate, np.float32).astype(np.float64)
    return 1.0 / (1.0 + np.exp(-z))


def combine(y_perm: np.ndarray, slot_row: np.ndarray, w: np.ndarray, T: int, k: int,
            y_shared: np.ndarray | None = None, gate: np.ndarray | None = None) -> np.ndarray:
    """Weighted un-permute: y[t] = sum over local slots j of w[t,j] * y_perm[slot_row[t*k+j]]
    (+ gate[t] * y_shared[t] for the always-active shared expert).  Tokens with no
    local expert get zeros (their contribution comes from other EP shards)."""
    H = y_perm.shape[1]
    y = np.zeros((T, H), np.float64)
    w = np.asarray(w, dtype=np.float64).reshape(T, k)
    for t in range(T):
        for j in range(k):
            r = int(slot_row[t * k + j])
            if r >= 0:
                y[t] += w[t, j] * y_perm[r]
    if y_shared is not None:
        g = np.ones(T) if gate is None else np.asarray(gate, np.float64)
        y += g[:, None] * np.asarray(y_shared, np.float64)
    return y


# --------------------------------------------------------------------------- sharding helpers
def tp_slice(w_gate, w_up, w_down, tp_degree: int, tp_rank: int):
    """Tensor-parallel shard p of E_t: rows [p*I_s,(p+1)*I_s) of gate and up, the same
    columns of down (I_s = I / E_t, E_t must divide I)."""
    I = w_gate.shape[1]
    if I % tp_degree:
        raise ValueError("E_t must divide the expert intermediate size")
    s = I // tp_degree
    sl = slice(tp_rank * s, (tp_rank + 1) * s)
    return w_gate[:, sl, :], w_up[:, sl, :], w_down[:, :, sl]


def ep_slice(w_gate, w_up, w_down, ep_degree: int, ep_rank: int):
    """Expert-parallel shard q of E_e: experts [q*E_loc,(q+1)*E_loc), contiguous.
    Returns (gate, up, down, n_local_experts, expert_offset)."""
    E = w_gate.shape[0]
    if E % ep_degree:
        raise ValueError("E_e must divide the number of experts")
    n = E // ep_degree
    sl = slice(ep_rank * n, (ep_rank + 1) * n)
    return w_gate[sl], w_up[sl], w_down[sl], n, ep_rank * n


# --------------------------------------------------------------------------- whole layer
def expert_layer(x_bits, logits, k, renorm, n_local_experts, expert_offset,
                 w_gate, w_up, w_down, shared=None, w_shared_gate=None, topk=None):
    """Route -> permute -> expert FFN -> combine on one shard; float64 [T,H].

    ``shared`` = (ws_gate, ws_up, ws_down) each with leading dim 1, applied to every
    token and scaled by sigmoid(x . w_shared_gate) when that vector is given.
    ``topk`` = (idx, w) overrides the routing step (used to evaluate a token sample
    against routing decisions taken elsewhere).
    """
    T = x_bits.shape[0]
    if topk is None:
        idx, _, w64 = route_topk(logits, k, renorm)
    else:
        idx, w64 = topk
    offs, row_src, slot_row, x_perm = permute(x_bits, idx, n_local_experts, expert_offset)
    y_perm = expert_ffn(x_perm, offs, w_gate, w_up, w_down)
    y_sh = gate = None
    if shared is not None:
        y_sh = expert_ffn(x_bits, np.array([0, T], np.int32), *shared)
        gate = shared_gate(x_bits, w_shared_gate) if w_shared_gate is not None else None
    return combine(y_perm, slot_row, w64, T, k, y_sh, gate)
