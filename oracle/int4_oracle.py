"""CPU oracle for the INT4 per-group backup of expert weights.

TEST INFRASTRUCTURE ONLY.  Slow, plain definition that the HIP quantise / dequantise kernels are
checked against.  It may be imported by tests, by the smoke check and by a benchmark's CPU
baseline leg, never by the product path; it shares no code with the HIP library.

What it computes (paper, "The Dynamic Parallelism Transition Strategy": a 4-bit quantised backup
of the expert weights is kept, uploaded, and dequantised to the native precision, BF16; of
per-tensor, per-channel and per-group quantisation the paper adopts per-group, and reports that
quantise-then-dequantise keeps more than 99.5 % cosine similarity to the original weights).  The
paper fixes neither the group size nor the code book; the format below is this repository's
reading, stated in its design notes: uniform affine ("asymmetric") quantisation of groups of 64
consecutive weights,

    scale = bf16((max - min) / 15),  code_i = clamp(rint((w_i - min) / scale), 0, 15),
    w'_i  = bf16(min + code_i * scale)

with min, max the group's extreme bf16 values.  Decisions that produce an integer (the code) and
the dequantised bf16 value are taken in float32, the precision of the kernels, so both sides can
be compared bit for bit; `dequantize_exact` gives the same affine map in float64 for the pins.

Layout: weights flat, n % 64 == 0; codes uint8 [n/2], element 2i in the low nibble of byte i and
element 2i+1 in the high nibble; qparams uint16 [n/64, 2] = bf16 bits of (scale, min).

Pins (tests/test_int4_oracle_pins.py): the paper's cosine-similarity figure on Gaussian weights;
the error bound |w - w'| <= scale/2 of round-to-nearest; brute-force nearest level on small
groups; exact reproduction of weights that already lie on 16 levels; code round trip; per-group
error no larger than per-tensor (the paper's ranking of the two); constant groups.
"""
from __future__ import annotations

import numpy as np

GROUP = 64
LEVELS = 15  # codes 0..15


def _bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _f32_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + (((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF))) >> np.uint32(16)).astype(np.uint16)


def quantize(w_bits: np.ndarray, group: int = GROUP):
    """bf16 bit patterns (any shape, size % group == 0) -> (codes uint8 [n/2], qparams uint16 [n/group, 2])."""
    w = _bf16_to_f32(np.asarray(w_bits).reshape(-1, group))
    mn = w.min(axis=1, keepdims=True)
    mx = w.max(axis=1, keepdims=True)
    scale_bits = _f32_to_bf16((mx - mn) / np.float32(LEVELS))
    scale = _bf16_to_f32(scale_bits)
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint((w - mn) / scale)           # float32 division and round-half-even, as the kernel
    q = np.where(scale > 0, q, np.float32(0))   # constant group: every weight is the minimum
    q = np.clip(q, 0, LEVELS).astype(np.uint8).reshape(-1)
    codes = (q[0::2] | (q[1::2] << np.uint8(4))).astype(np.uint8)
    qparams = np.concatenate([scale_bits, _f32_to_bf16(mn)], axis=1).astype(np.uint16)
    return codes, qparams


def unpack_codes(codes: np.ndarray) -> np.ndarray:
    c = np.asarray(codes, dtype=np.uint8)
    out = np.empty(c.size * 2, dtype=np.uint8)
    out[0::2] = c & np.uint8(15)
    out[1::2] = c >> np.uint8(4)
    return out


def dequantize(codes: np.ndarray, qparams: np.ndarray, group: int = GROUP) -> np.ndarray:
    """-> bf16 bit patterns [n]: bf16(min + code * scale), the sum rounded once to float32 first."""
    q = unpack_codes(codes).reshape(-1, group).astype(np.float32)
    scale = _bf16_to_f32(qparams[:, 0:1])
    mn = _bf16_to_f32(qparams[:, 1:2])
    return _f32_to_bf16(q * scale + mn).reshape(-1)   # code * scale is exact in float32 (4 + 8 bits)


def dequantize_exact(codes: np.ndarray, qparams: np.ndarray, group: int = GROUP) -> np.ndarray:
    """The affine map min + code * scale in float64, not rounded."""
    q = unpack_codes(codes).reshape(-1, group).astype(np.float64)
    return (q * _bf16_to_f32(qparams[:, 0:1]).astype(np.float64) + _bf16_to_f32(qparams[:, 1:2]).astype(np.float64)).reshape(-1)


def quantize_per_tensor(w_bits: np.ndarray):
    """The per-tensor scheme the paper compares against: one (scale, min) for the whole tensor."""
    return quantize(np.asarray(w_bits).reshape(-1), group=np.asarray(w_bits).size)


def cosine_similarity(a_bits: np.ndarray, b_bits: np.ndarray) -> float:
    a = _bf16_to_f32(np.asarray(a_bits).reshape(-1)).astype(np.float64)
    b = _bf16_to_f32(np.asarray(b_bits).reshape(-1)).astype(np.float64)
    return float(a @ b / np.sqrt((a @ a) * (b @ b)))
