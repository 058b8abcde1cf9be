"""GPU parity of the INT4 per-group kernels against the CPU oracle, through the C ABI.
Codes, group parameters and dequantised bf16 values are all compared bit for bit: every decision is
taken in float32 with round-to-nearest-even on both sides."""
import numpy as np
import pytest
import torch

from oracle import int4_oracle as Q
from paper_2508_19373_amd import binding as B
from paper_2508_19373_amd import inputs as I
from paper_2508_19373_amd.layer import bf16_bits, bf16_tensor

pytestmark = pytest.mark.gpu


def _weights(n, seed=0, sigma=0.02):
    rng = np.random.Generator(np.random.Philox(seed))
    return I.f32_to_bf16_bits((sigma * rng.standard_normal(n)).astype(np.float32))


def _gpu_quantize(w_bits):
    n = w_bits.size
    w = bf16_tensor(w_bits)
    codes = torch.full((max(n // 2, 1),), 0xAB, dtype=torch.uint8, device="cuda")
    qp = torch.full((max(n // 64, 1), 2), 0x7FC0, dtype=torch.int16, device="cuda")
    B.moe_int4_quantize(w, n, codes, qp)
    torch.cuda.synchronize()
    return codes[:n // 2].cpu().numpy(), qp[:n // 64].cpu().numpy().view(np.uint16)


def _gpu_dequantize(codes, qparams, n):
    c = torch.from_numpy(np.ascontiguousarray(codes)).cuda() if n else torch.zeros(16, dtype=torch.uint8, device="cuda")
    p = torch.from_numpy(np.ascontiguousarray(qparams).view(np.int16)).cuda() if n else torch.zeros((1, 2), dtype=torch.int16, device="cuda")
    out = torch.full((max(n, 8),), -1.0, dtype=torch.bfloat16, device="cuda")
    B.moe_int4_dequantize(c, p, n, out)
    torch.cuda.synchronize()
    return bf16_bits(out)


@pytest.mark.parametrize("n", [64, 192, 8192, 8192 + 64, 3 * 8192 - 64, (1 << 20) + 5 * 64])
def test_quantize_and_dequantize_bit_exact(n):
    w = _weights(n, seed=n % 97)
    codes, qp = _gpu_quantize(w)
    ref_codes, ref_qp = Q.quantize(w)
    assert np.array_equal(qp, ref_qp)
    assert np.array_equal(codes, ref_codes)
    got = _gpu_dequantize(ref_codes, ref_qp, n)
    assert np.array_equal(got[:n], Q.dequantize(ref_codes, ref_qp))
    if n >= 8:
        assert np.all(got[n:] == bf16_bits(torch.full((1,), -1.0, dtype=torch.bfloat16))[0])  # nothing past the end


def test_dequantize_arbitrary_codes_and_parameters():
    rng = np.random.default_rng(5)
    n = 64 * 777
    codes = rng.integers(0, 256, n // 2, dtype=np.uint8)
    scale = I.f32_to_bf16_bits(rng.uniform(0, 0.1, n // 64).astype(np.float32))
    mn = I.f32_to_bf16_bits(rng.normal(0, 1, n // 64).astype(np.float32))
    qp = np.stack([scale, mn], axis=1).astype(np.uint16)
    assert np.array_equal(_gpu_dequantize(codes, qp, n)[:n], Q.dequantize(codes, qp))


def test_special_groups():
    const = np.full(64, 0.375, dtype=np.float32)
    two = np.where(np.arange(64) % 3 == 0, -1.0, 2.0).astype(np.float32)
    levels = (-0.5 + ((np.arange(64) * 7) % 16) / 16.0).astype(np.float32)
    zeros = np.zeros(64, dtype=np.float32)
    big = (np.arange(64) - 30).astype(np.float32) * 1000.0
    w = I.f32_to_bf16_bits(np.concatenate([const, two, levels, zeros, big]))
    codes, qp = _gpu_quantize(w)
    ref_codes, ref_qp = Q.quantize(w)
    assert np.array_equal(codes, ref_codes) and np.array_equal(qp, ref_qp)
    back = _gpu_dequantize(codes, qp, w.size)[:w.size]
    assert np.array_equal(back, Q.dequantize(ref_codes, ref_qp))
    assert np.array_equal(back[:64], w[:64]) and np.array_equal(back[128:256], w[128:256])  # exact cases


def test_empty_tensor_is_a_no_op():
    out = _gpu_dequantize(np.zeros(0, np.uint8), np.zeros((0, 2), np.uint16), 0)
    assert np.all(I.bf16_bits_to_f32(out) == -1.0)


def test_full_size_expert_matrix_round_trip():
    # one Mixtral-8x7B expert matrix: 14336 x 4096 weights, the unit the switching path dequantises
    shape = I.MoEShape("one-expert", 4096, 1, 1, 14336, True)
    wg, _, _ = I.make_expert_weights(0, shape)
    w = wg.reshape(-1)
    n = w.size
    wt = bf16_tensor(w)
    codes = torch.empty(n // 2, dtype=torch.uint8, device="cuda")
    qp = torch.empty((n // 64, 2), dtype=torch.int16, device="cuda")
    back = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    B.moe_int4_quantize(wt, n, codes, qp)
    B.moe_int4_dequantize(codes, qp, n, back)
    torch.cuda.synchronize()
    # the paper's figure, computed over the whole matrix on the device (plain float64 reductions of the outputs)
    a, b = wt.double(), back.double()
    cos = float((a @ b) / torch.sqrt((a @ a) * (b @ b)))
    assert cos > 0.995
    # sampled groups against the oracle, bit for bit
    rng = np.random.default_rng(2)
    groups = np.unique(np.concatenate([[0, n // 64 - 1], rng.integers(0, n // 64, 4000)]))
    c_host, p_host, b_host = codes.cpu().numpy(), qp.cpu().numpy().view(np.uint16), bf16_bits(back)
    sel = (groups[:, None] * 64 + np.arange(64)[None, :]).reshape(-1)
    ref_codes, ref_qp = Q.quantize(w[sel])
    assert np.array_equal(p_host[groups], ref_qp)
    assert np.array_equal(c_host.reshape(-1, 32)[groups].reshape(-1), ref_codes)
    assert np.array_equal(b_host[sel], Q.dequantize(ref_codes, ref_qp))
