"""Seeded input generators: reproducible, element-addressable, right distributions."""
import numpy as np

from paper_2508_19373_amd import inputs as I


def test_bf16_encode_is_round_to_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, 1.005, -2.5, 0.0], np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie between 0x3F80 and 0x3F81 -> even (0x3F80)
    # 1.01171875 = 1 + 3*2^-8 is a tie between 0x3F81 and 0x3F82 -> even (0x3F82)
    bits = I.f32_to_bf16_bits(f)
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x0000]
    assert np.array_equal(I.f32_to_bf16_bits(I.bf16_bits_to_f32(bits)), bits)


def test_bf16_encode_matches_torch():
    import torch
    f = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    t = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(I.f32_to_bf16_bits(f), t)


def test_reproducible_and_prefix_property():
    a = I.make_layer_inputs(I.TINY, 64, 0)
    b = I.make_layer_inputs(I.TINY, 64, 0)
    c = I.make_layer_inputs(I.TINY, 64, 1)
    assert np.array_equal(a.x, b.x) and np.array_equal(a.w_gate, b.w_gate)
    assert not np.array_equal(a.x, c.x) and not np.array_equal(a.w_down, c.w_down)
    assert np.array_equal(I.make_x(0, 16, 512), a.x[:16])
    assert a.w_gate.shape == (8, 1024, 512) and a.w_down.shape == (8, 512, 1024)
    assert a.w_router.shape == (512, 8) and a.w_router.dtype == np.float32


def test_distributions():
    a = I.make_layer_inputs(I.TINY, 64, 0)
    x = I.bf16_bits_to_f32(a.x)
    assert abs(x.mean()) < 0.02 and abs(x.std() - 1.0) < 0.02
    w = I.bf16_bits_to_f32(a.w_up)
    assert abs(w.mean()) < 1e-4 and abs(w.std() - 0.02) < 2e-4
    wr = I.make_router_weight(0, I.MIXTRAL)
    assert abs(wr.std() - 0.02) < 5e-4 and np.abs(wr).max() <= 0.02 * 3 ** 0.5 + 1e-7


def test_zipf_logits_first_choice_frequencies():
    L = I.make_zipf_logits(0, 40000, 8)
    p = I.zipf_popularity(8)
    freq = np.bincount(L.argmax(1), minlength=8) / 40000
    assert np.abs(freq - p).max() < 0.01
    assert abs(p[0] - 0.4286) < 1e-3 and abs(p[7] - 0.0353) < 1e-3


def test_ep_and_tp_shards_are_slices_of_one_model():
    s = I.MoEShape("s", 64, 8, 2, 128, True)
    g, u, d = I.make_expert_weights(0, s)
    g2, u2, d2 = I.make_expert_weights(0, s.shard(tp_degree=2, tp_rank=1, ep_degree=4, ep_rank=2))
    assert np.array_equal(g2, g[4:6, 64:128]) and np.array_equal(u2, u[4:6, 64:128])
    assert np.array_equal(d2, d[4:6, :, 64:128])


def test_shared_gate_weight_is_bf16_representable():
    w = I.make_shared_gate_weight(0, 2048)
    assert np.array_equal(I.bf16_bits_to_f32(I.f32_to_bf16_bits(w)), w)
