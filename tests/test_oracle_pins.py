"""Pins for the CPU oracle: each check ties an oracle function to something other
than itself -- brute force over all experts, a library routine, a closed form or an
invariant of the method (TP partial sums add up, EP shard outputs add up)."""
import math

import numpy as np
import pytest
import scipy.special

from oracle import moe_oracle as O
from paper_2508_19373_amd import inputs as I

SMALL = I.MoEShape("small", 64, 8, 2, 128, True)


def _inputs(shape=SMALL, T=24, seed=0):
    li = I.make_layer_inputs(shape, T, seed)
    logits = li.logits if li.logits is not None else O.router_logits(li.x, li.w_router)
    return li, logits


def _dense_bruteforce(li, logits, k, renorm, experts=None):
    """Evaluate every expert on every token (no permutation, no grouping), then mix
    with a dense [T,E] weight matrix that is zero except at the k selected experts."""
    x = I.bf16_bits_to_f32(li.x).astype(np.float64)
    T, E = logits.shape
    p = scipy.special.softmax(logits.astype(np.float64), axis=1)
    dense_w = np.zeros((T, E))
    for t in range(T):
        chosen = np.lexsort((np.arange(E), -logits[t].astype(np.float64)))[:k]
        dense_w[t, chosen] = p[t, chosen] / (p[t, chosen].sum() if renorm else 1.0)
    y = np.zeros((T, x.shape[1]))
    experts = range(E) if experts is None else experts
    for le, e in enumerate(experts):
        Wg = I.bf16_bits_to_f32(li.w_gate[le]).astype(np.float64)
        Wu = I.bf16_bits_to_f32(li.w_up[le]).astype(np.float64)
        Wd = I.bf16_bits_to_f32(li.w_down[le]).astype(np.float64)
        for t in range(T):
            g = Wg @ x[t]
            u = Wu @ x[t]
            h = g * scipy.special.expit(g) * u
            y[t] += dense_w[t, e] * (Wd @ h)
    return y


def _rel(a, b):
    return np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300)


def test_bf16_decode_matches_struct_definition():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3DCD ~ 0.1 (bf16), 0x0000 = 0
    bits = np.array([0x3F80, 0xC000, 0x3DCD, 0x0000, 0x4049], np.uint16)
    want = [1.0, -2.0, 0.10009765625, 0.0, 3.140625]
    assert O.bf16_to_f64(bits).tolist() == want


@pytest.mark.parametrize("renorm", [True, False])
@pytest.mark.parametrize("k", [1, 2, 3])
def test_layer_equals_dense_bruteforce(k, renorm):
    li, logits = _inputs()
    y = O.expert_layer(li.x, logits, k, renorm, 8, 0, li.w_gate, li.w_up, li.w_down)
    yb = _dense_bruteforce(li, logits, k, renorm)
    assert _rel(y, yb) < 1e-12
    assert np.abs(yb).max() > 1e-4  # not trivially zero


@pytest.mark.parametrize("tp", [1, 2, 4, 8])
def test_tp_partial_sums_add_to_unsharded(tp):
    li, logits = _inputs()
    full = O.expert_layer(li.x, logits, 2, True, 8, 0, li.w_gate, li.w_up, li.w_down)
    acc = np.zeros_like(full)
    for p in range(tp):
        g, u, d = O.tp_slice(li.w_gate, li.w_up, li.w_down, tp, p)
        assert g.shape[1] == SMALL.inter // tp and d.shape[2] == SMALL.inter // tp
        acc += O.expert_layer(li.x, logits, 2, True, 8, 0, g, u, d)
    assert _rel(acc, full) < 1e-12
    # the generator's own shard slicing agrees with slicing the full weights
    for p in range(tp):
        sg, su, sd = I.make_expert_weights(0, SMALL.shard(tp_degree=tp, tp_rank=p))
        g, u, d = O.tp_slice(li.w_gate, li.w_up, li.w_down, tp, p)
        assert np.array_equal(sg, g) and np.array_equal(su, u) and np.array_equal(sd, d)


def test_tp_slice_rejects_non_divisor():
    li, _ = _inputs()
    with pytest.raises(ValueError):
        O.tp_slice(li.w_gate, li.w_up, li.w_down, 3, 0)
    with pytest.raises(ValueError):
        O.ep_slice(li.w_gate, li.w_up, li.w_down, 3, 0)


@pytest.mark.parametrize("ep", [1, 2, 4, 8])
def test_ep_shard_outputs_add_to_full_layer(ep):
    li, logits = _inputs()
    full = O.expert_layer(li.x, logits, 2, True, 8, 0, li.w_gate, li.w_up, li.w_down)
    idx, _, _ = O.route_topk(logits, 2, True)
    acc = np.zeros_like(full)
    rows = 0
    for q in range(ep):
        g, u, d, n, off = O.ep_slice(li.w_gate, li.w_up, li.w_down, ep, q)
        assert (n, off) == (8 // ep, q * (8 // ep))
        acc += O.expert_layer(li.x, logits, 2, True, n, off, g, u, d)
        offs, *_ = O.permute(li.x, idx, n, off)
        rows += int(offs[-1])
        # each shard equals the brute force restricted to its experts
        li_q = I.make_layer_inputs(SMALL.shard(ep_degree=ep, ep_rank=q), 24, 0)
        assert np.array_equal(li_q.w_gate, g)
        yb = _dense_bruteforce(li_q, logits, 2, True, experts=range(off, off + n))
        yq = O.expert_layer(li.x, logits, 2, True, n, off, g, u, d)
        assert _rel(yq, yb) < 1e-12 or np.abs(yb).max() == 0
    assert rows == 24 * 2
    assert _rel(acc, full) < 1e-12


def test_hybrid_ep_tp_shards_add_to_full_layer():
    li, logits = _inputs()
    full = O.expert_layer(li.x, logits, 2, True, 8, 0, li.w_gate, li.w_up, li.w_down)
    acc = np.zeros_like(full)
    for q in range(2):
        g, u, d, n, off = O.ep_slice(li.w_gate, li.w_up, li.w_down, 2, q)
        for p in range(2):
            gs, us, ds = O.tp_slice(g, u, d, 2, p)
            acc += O.expert_layer(li.x, logits, 2, True, n, off, gs, us, ds)
    assert _rel(acc, full) < 1e-12


# ------------------------------------------------------------------ routing pins
def test_topk_all_equal_logits_pins_tiebreak():
    L = np.zeros((3, 8), np.float32)
    idx, w, _ = O.route_topk(L, 3, True)
    assert idx.tolist() == [[0, 1, 2]] * 3
    assert np.allclose(w, 1.0 / 3.0, rtol=0, atol=1e-7)
    idx, w, _ = O.route_topk(L, 3, False)
    assert idx.tolist() == [[0, 1, 2]] * 3
    assert np.allclose(w, 1.0 / 8.0, rtol=0, atol=1e-7)


def test_topk_signed_zero_and_partial_ties():
    L = np.array([[0.0, -0.0, 1.0, 1.0, -1.0],
                  [-0.0, 0.0, -5.0, -5.0, -5.0],
                  [2.0, 3.0, 3.0, 2.0, 3.0]], np.float32)
    idx, _, _ = O.route_topk(L, 4, True)
    assert idx.tolist() == [[2, 3, 0, 1], [0, 1, 2, 3], [1, 2, 4, 0]]


def test_topk_hand_worked_example():
    # logits ln1, ln2, ln3, ln4 -> softmax = (1,2,3,4)/10
    L = np.log(np.array([[1.0, 2.0, 3.0, 4.0]])).astype(np.float32)
    idx, w, w64 = O.route_topk(L, 2, False)
    assert idx.tolist() == [[3, 2]]
    assert np.allclose(w64, [[0.4, 0.3]], atol=1e-7)
    idx, w, w64 = O.route_topk(L, 2, True)
    assert np.allclose(w64, [[4 / 7, 3 / 7]], atol=1e-7)


@pytest.mark.parametrize("renorm", [True, False])
def test_topk_against_library_softmax_and_argsort(renorm):
    rng = np.random.default_rng(5)
    L = rng.standard_normal((200, 60)).astype(np.float32)  # tie-free with probability 1
    k = 4
    idx, w, w64 = O.route_topk(L, k, renorm)
    lib_order = np.argsort(-L.astype(np.float64), axis=1, kind="stable")[:, :k]
    assert np.array_equal(idx, lib_order.astype(np.int32))
    p = scipy.special.softmax(L.astype(np.float64), axis=1)
    mass = np.take_along_axis(p, lib_order, axis=1)
    if renorm:
        assert np.allclose(w64.sum(1), 1.0, atol=1e-15)
        # renormalised weights equal a softmax over just the k selected logits
        sel = np.take_along_axis(L.astype(np.float64), lib_order, axis=1)
        assert np.allclose(w64, scipy.special.softmax(sel, axis=1), atol=1e-14)
    else:
        assert np.allclose(w64, mass, atol=1e-15)
        assert np.all(w64.sum(1) <= 1.0 + 1e-15)
    assert np.all(w64 >= 0) and np.all(np.diff(w64, axis=1) <= 0)
    assert w.dtype == np.float32 and np.allclose(w, w64, rtol=1e-7)


def test_topk_k_equals_E_is_plain_softmax():
    rng = np.random.default_rng(7)
    L = rng.standard_normal((10, 8)).astype(np.float32)
    idx, _, w64 = O.route_topk(L, 8, False)
    p = np.zeros((10, 8))
    np.put_along_axis(p, idx.astype(np.int64), w64, axis=1)
    assert np.allclose(p, scipy.special.softmax(L.astype(np.float64), axis=1), atol=1e-15)


def test_topk_large_logits_no_overflow():
    L = np.array([[1000.0, 999.0, -1000.0]], np.float32)
    _, _, w64 = O.route_topk(L, 2, False)
    e = math.exp(-1.0)
    assert np.allclose(w64, [[1 / (1 + e), e / (1 + e)]], atol=1e-12)


def test_topk_rejects_nonfinite_and_bad_k():
    with pytest.raises(ValueError):
        O.route_topk(np.array([[0.0, np.nan]], np.float32), 1, True)
    with pytest.raises(ValueError):
        O.route_topk(np.zeros((1, 4), np.float32), 5, True)


def test_router_logits_against_exact_rational_arithmetic():
    from fractions import Fraction
    li, _ = _inputs(T=3)
    L = O.router_logits(li.x, li.w_router)
    x = I.bf16_bits_to_f32(li.x)
    for t in range(3):
        for e in (0, 5):
            exact = sum(Fraction(float(x[t, h])) * Fraction(float(li.w_router[h, e])) for h in range(64))
            assert L[t, e] == np.float32(float(exact))


# ------------------------------------------------------------------ permutation pins
@pytest.mark.parametrize("n_local,off", [(8, 0), (2, 0), (2, 6), (4, 4), (1, 3)])
def test_permute_equals_library_stable_sort(n_local, off):
    rng = np.random.default_rng(11)
    T, k, E, H = 50, 3, 8, 16
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    x = I.make_x(1, T, H)
    offs, row_src, slot_row, x_perm = O.permute(x, idx, n_local, off)
    flat = idx.reshape(-1)
    local = np.nonzero((flat >= off) & (flat < off + n_local))[0]
    order = local[np.argsort(flat[local], kind="stable")]
    assert np.array_equal(row_src, order.astype(np.int32))
    R = len(local)
    assert offs[0] == 0 and offs[-1] == R and np.all(np.diff(offs) >= 0)
    assert np.array_equal(np.diff(offs), np.bincount(flat[local] - off, minlength=n_local))
    assert np.array_equal(slot_row[row_src], np.arange(R))
    assert np.all(slot_row[np.setdiff1d(np.arange(T * k), local)] == -1)
    for e in range(n_local):
        seg = row_src[offs[e]:offs[e + 1]]
        assert np.all(np.diff(seg) > 0) and np.all(flat[seg] == e + off)
    assert np.array_equal(x_perm, x[row_src // k])


def test_permute_empty_shard_and_empty_batch():
    x = I.make_x(0, 4, 8)
    idx = np.array([[0, 1]] * 4, np.int32)
    offs, row_src, slot_row, x_perm = O.permute(x, idx, 2, 6)
    assert offs.tolist() == [0, 0, 0] and len(row_src) == 0 and x_perm.shape == (0, 8)
    assert np.all(slot_row == -1)
    offs, row_src, slot_row, x_perm = O.permute(x[:0], idx[:0], 2, 0)
    assert offs.tolist() == [0, 0, 0] and slot_row.shape == (0,)


# ------------------------------------------------------------------ expert FFN / combine pins
def test_single_expert_reduces_to_three_matmul_mlp():
    shape = I.MoEShape("mlp", 64, 1, 1, 128, True)
    li = I.make_layer_inputs(shape, 9, 3)
    y = O.expert_layer(li.x, np.zeros((9, 1), np.float32), 1, True, 1, 0, li.w_gate, li.w_up, li.w_down)
    x = I.bf16_bits_to_f32(li.x).astype(np.float64)
    Wg, Wu, Wd = (I.bf16_bits_to_f32(w[0]).astype(np.float64) for w in (li.w_gate, li.w_up, li.w_down))
    g = np.einsum("th,ih->ti", x, Wg)
    u = np.einsum("th,ih->ti", x, Wu)
    ref = np.einsum("ti,ni->tn", g * scipy.special.expit(g) * u, Wd)
    assert _rel(y, ref) < 1e-13


def test_silu_known_values():
    z = np.array([0.0, 1.0, -1.0, 20.0])
    want = [0.0, 1 / (1 + math.exp(-1)), -1 / (1 + math.exp(1)), 20 / (1 + math.exp(-20))]
    assert np.allclose(O.silu(z), want, atol=1e-15)


def test_ffn_linear_in_down_and_zero_gate():
    li, logits = _inputs()
    idx, _, _ = O.route_topk(logits, 2, True)
    offs, _, _, xp = O.permute(li.x, idx, 8, 0)
    y1 = O.expert_ffn(xp, offs, li.w_gate, li.w_up, li.w_down)
    # bf16 bit pattern with the exponent field bumped by one doubles every weight exactly
    wd2 = (li.w_down + np.uint16(0x0080)).astype(np.uint16)
    y2 = O.expert_ffn(xp, offs, li.w_gate, li.w_up, wd2)
    assert _rel(y2, 2 * y1) < 1e-15
    y0 = O.expert_ffn(xp, offs, np.zeros_like(li.w_gate), li.w_up, li.w_down)
    assert np.all(y0 == 0)
    # swapping gate and up must change the result (silu is applied to gate only)
    ysw = O.expert_ffn(xp, offs, li.w_up, li.w_gate, li.w_down)
    assert _rel(ysw, y1) > 1e-2


def test_identical_experts_with_k_equal_E_give_the_single_expert():
    shape = I.MoEShape("same", 64, 4, 4, 128, True)
    li = I.make_layer_inputs(shape, 7, 2)
    for w in (li.w_gate, li.w_up, li.w_down):
        w[1:] = w[0]
    logits = O.router_logits(li.x, li.w_router)
    y = O.expert_layer(li.x, logits, 4, True, 4, 0, li.w_gate, li.w_up, li.w_down)
    one = O.expert_ffn(li.x, np.array([0, 7], np.int32), li.w_gate[:1], li.w_up[:1], li.w_down[:1])
    assert _rel(y, one) < 1e-13


def test_token_permutation_equivariance():
    li, logits = _inputs()
    perm = np.random.default_rng(3).permutation(24)
    y = O.expert_layer(li.x, logits, 2, True, 8, 0, li.w_gate, li.w_up, li.w_down)
    yp = O.expert_layer(li.x[perm], logits[perm], 2, True, 8, 0, li.w_gate, li.w_up, li.w_down)
    assert _rel(yp, y[perm]) < 1e-13


def test_shared_expert_gate_half_when_ws_zero_and_additivity():
    shape = I.MoEShape("sh", 64, 8, 2, 128, False, inter_shared=256)
    li = I.make_layer_inputs(shape, 12, 4)
    logits = O.router_logits(li.x, li.w_router)
    shared = (li.ws_gate, li.ws_up, li.ws_down)
    assert np.all(O.shared_gate(li.x, np.zeros(64, np.float32)) == 0.5)
    routed = O.expert_layer(li.x, logits, 2, False, 8, 0, li.w_gate, li.w_up, li.w_down)
    ysh = O.expert_ffn(li.x, np.array([0, 12], np.int32), *shared)
    both0 = O.expert_layer(li.x, logits, 2, False, 8, 0, li.w_gate, li.w_up, li.w_down,
                           shared=shared, w_shared_gate=np.zeros(64, np.float32))
    assert _rel(both0, routed + 0.5 * ysh) < 1e-14
    both = O.expert_layer(li.x, logits, 2, False, 8, 0, li.w_gate, li.w_up, li.w_down,
                          shared=shared, w_shared_gate=li.w_shared_gate)
    x = I.bf16_bits_to_f32(li.x).astype(np.float64)
    gate = scipy.special.expit(x @ li.w_shared_gate.astype(np.float64))
    assert _rel(both, routed + gate[:, None] * ysh) < 1e-14
    assert 0.02 < gate.std()  # the gate actually varies


def test_combine_zero_for_tokens_without_local_expert():
    y_perm = np.arange(6, dtype=np.float64).reshape(2, 3) + 1
    slot_row = np.array([-1, 0, -1, -1, 1, -1], np.int32)
    w = np.array([[0.5, 0.25], [0.7, 0.3], [0.6, 0.4]])
    y = O.combine(y_perm, slot_row, w, 3, 2)
    assert np.allclose(y, [[0.25, 0.5, 0.75], [0, 0, 0], [2.4, 3.0, 3.6]])


def _dense_mix(li, idx, w, experts_lo=0, n_local=None):
    """sum_j w[t,j] * FFN_{idx[t,j]}(x_t) over the local experts, token by token, from hand-made
    routing decisions (no logits, no softmax, no permutation)."""
    x = I.bf16_bits_to_f32(li.x).astype(np.float64)
    n_local = li.w_gate.shape[0] if n_local is None else n_local
    y = np.zeros((x.shape[0], x.shape[1]))
    for t in range(x.shape[0]):
        for j in range(idx.shape[1]):
            le = int(idx[t, j]) - experts_lo
            if 0 <= le < n_local:
                Wg = I.bf16_bits_to_f32(li.w_gate[le]).astype(np.float64)
                Wu = I.bf16_bits_to_f32(li.w_up[le]).astype(np.float64)
                Wd = I.bf16_bits_to_f32(li.w_down[le]).astype(np.float64)
                g = Wg @ x[t]
                y[t] += w[t, j] * (Wd @ (g * scipy.special.expit(g) * (Wu @ x[t])))
    return y


@pytest.mark.parametrize("renorm", [True, False])
def test_layer_with_given_routing_equals_routed_call(renorm):
    # the routing override is the branch the full-size GPU checks take: feeding it the decisions
    # route_topk makes from the same logits must reproduce the routed call exactly, also on a
    # token sample (each output row depends on its own token only) and on an expert-parallel shard
    li, logits = _inputs(T=40)
    idx, _, w64 = O.route_topk(logits, 3, renorm)
    a = O.expert_layer(li.x, logits, 3, renorm, 8, 0, li.w_gate, li.w_up, li.w_down)
    b = O.expert_layer(li.x, None, 3, renorm, 8, 0, li.w_gate, li.w_up, li.w_down, topk=(idx, w64))
    assert np.array_equal(a, b)
    sel = np.array([0, 3, 4, 17, 39])
    c = O.expert_layer(li.x[sel], None, 3, renorm, 8, 0, li.w_gate, li.w_up, li.w_down, topk=(idx[sel], w64[sel]))
    assert _rel(c, a[sel]) < 1e-13
    g, u, d, n, off = O.ep_slice(li.w_gate, li.w_up, li.w_down, 4, 2)
    e1 = O.expert_layer(li.x, logits, 3, renorm, n, off, g, u, d)
    e2 = O.expert_layer(li.x[sel], None, 3, renorm, n, off, g, u, d, topk=(idx[sel], w64[sel]))
    assert _rel(e2, e1[sel]) < 1e-13


def test_layer_with_handmade_routing_equals_dense_mix():
    # decisions no softmax would produce (weights that do not sum to one, a negative one, repeated
    # use of one expert by neighbouring tokens): the override must take them as given
    li, _ = _inputs(T=12)
    rng = np.random.default_rng(5)
    idx = np.stack([rng.permutation(8)[:2] for _ in range(12)]).astype(np.int32)
    idx[3] = idx[4] = idx[5] = (7, 0)
    w = rng.uniform(-0.5, 1.5, size=(12, 2))
    y = O.expert_layer(li.x, None, 2, False, 8, 0, li.w_gate, li.w_up, li.w_down, topk=(idx, w))
    assert _rel(y, _dense_mix(li, idx, w)) < 1e-12
    # swapping the two slots of every token changes nothing but the summation order
    y2 = O.expert_layer(li.x, None, 2, False, 8, 0, li.w_gate, li.w_up, li.w_down, topk=(idx[:, ::-1], w[:, ::-1]))
    assert _rel(y2, y) < 1e-13
    # an expert-parallel shard keeps only its experts' terms
    g, u, d, n, off = O.ep_slice(li.w_gate, li.w_up, li.w_down, 2, 1)
    ys = O.expert_layer(li.x, None, 2, False, n, off, g, u, d, topk=(idx, w))
    li_s = type("S", (), {"x": li.x, "w_gate": g, "w_up": u, "w_down": d})
    assert _rel(ys, _dense_mix(li_s, idx, w, experts_lo=off, n_local=n)) < 1e-12
