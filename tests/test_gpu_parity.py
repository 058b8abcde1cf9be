"""GPU parity: every step of the HIP path against the CPU oracle, through the C ABI, on the
same seeded inputs.  Integer outputs (top-k ids, offsets, permutation, permuted rows) must be
bit-exact given identical fp32 logits; floating-point outputs must be within rel-L2 5e-3 and
max-abs 2e-2 (the latter applied to the fp32-output path on Mixtral-scale outputs, whose bf16
spacing alone reaches 2^-4)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2508_19373_amd import binding as B
from paper_2508_19373_amd import inputs as I
from guards import Guards
from paper_2508_19373_amd.layer import ExpertShardLayer, bf16_bits, bf16_tensor

pytestmark = pytest.mark.gpu

REL_L2 = 5e-3
MAX_ABS = 2e-2


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def _rel(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def _route_gpu(x_bits, w_router, logits, T, H, E, k, renorm):
    g = Guards()
    d_logits = g.empty((max(T, 1), E), torch.float32)
    idx = g.empty((max(T, 1), k), torch.int32, fill=-7)
    w = g.empty((max(T, 1), k), torch.float32)
    flags = B.MOE_RENORM_TOPK if renorm else 0
    if logits is not None:
        d_logits[:T].copy_(_dev(logits))
        flags |= B.MOE_LOGITS_GIVEN
        B.moe_route_topk(None, None, d_logits, T, H, E, k, flags, idx, w)
    else:
        B.moe_route_topk(bf16_tensor(x_bits), _dev(w_router), d_logits, T, H, E, k, flags, idx, w)
    g.check()
    return d_logits[:T].cpu().numpy(), idx[:T].cpu().numpy(), w[:T].cpu().numpy()


# ------------------------------------------------------------------ route
@pytest.mark.parametrize("shape,T", [(I.TINY, 64), (I.MoEShape("q", 256, 60, 4, 128, False), 77),
                                     (I.MoEShape("wide", 128, 200, 6, 128, True), 33),
                                     (I.MoEShape("odd", 64, 13, 3, 128, True), 5),
                                     # up to 16 experts: W_r goes through the wavefronts' LDS areas
                                     (I.MoEShape("e3", 96, 3, 2, 128, True), 37),
                                     (I.MoEShape("e9", 4096, 9, 2, 128, True), 16),
                                     (I.MoEShape("e16", 2080, 16, 4, 128, False), 150),
                                     (I.MoEShape("e8", 4096, 8, 2, 128, True), 1),
                                     # up to 64 tokens with 8 experts: one workgroup per token on the vector units
                                     (I.MoEShape("e8s", 4096, 8, 2, 128, True), 64),
                                     (I.MoEShape("e16s", 2080, 16, 4, 128, False), 40),
                                     (I.MoEShape("e16t", 72, 16, 16, 128, True), 3),
                                     (I.MoEShape("max", 192, 256, 16, 128, False), 40),    # E and k at their limits
                                     # more than 128 tokens: logits and selection in one kernel, 2 to 16 expert tiles
                                     (I.MoEShape("q2", 256, 30, 4, 128, False), 300),
                                     (I.MoEShape("q4", 256, 60, 4, 128, False), 333),
                                     (I.MoEShape("q8", 128, 100, 6, 128, True), 200),
                                     (I.MoEShape("q16", 128, 200, 6, 128, True), 300)])
def test_route_logits_and_topk(shape, T):
    li = I.make_layer_inputs(shape, T, 0, weights=False)
    E, k = shape.n_experts, shape.top_k
    logits, idx, w = _route_gpu(li.x, li.w_router, None, T, shape.hidden, E, k, shape.renorm)
    ref_logits = O.router_logits(li.x, li.w_router).astype(np.float64)
    assert np.all(np.abs(logits - ref_logits) <= 1e-5 * (1 + np.abs(ref_logits)))
    # identical fp32 logits in, identical integer decisions out
    ridx, rw, _ = O.route_topk(logits, k, shape.renorm)
    assert np.array_equal(idx, ridx)
    assert np.allclose(w, rw, rtol=2e-6, atol=1e-9)


@pytest.mark.parametrize("renorm", [True, False])
def test_route_given_logits_with_ties(renorm):
    rng = np.random.default_rng(1)
    L = rng.integers(-2, 3, size=(300, 60)).astype(np.float32)  # many exact ties
    L[0, :] = 0.0
    L[1, :] = -0.0
    L[1, 5] = 0.0
    L[2, :] = np.where(np.arange(60) % 2 == 0, -0.0, 0.0)
    logits, idx, w = _route_gpu(None, None, L, 300, 0, 60, 4, renorm)
    assert np.array_equal(logits, L)
    ridx, rw, _ = O.route_topk(L, 4, renorm)
    assert np.array_equal(idx, ridx)
    assert idx[0].tolist() == [0, 1, 2, 3] and idx[1].tolist() == [0, 1, 2, 3]
    assert np.allclose(w, rw, rtol=2e-6, atol=1e-9)


def test_route_zipf_logits_k_equals_E_and_empty_batch():
    L = I.make_zipf_logits(3, 50, 8)
    _, idx, w = _route_gpu(None, None, L, 50, 0, 8, 8, False)
    ridx, rw, _ = O.route_topk(L, 8, False)
    assert np.array_equal(idx, ridx) and np.allclose(w, rw, rtol=2e-6)
    assert np.allclose(w.sum(1), 1.0, atol=1e-6)
    _route_gpu(None, None, np.zeros((0, 8), np.float32), 0, 0, 8, 2, True)  # T = 0 is a no-op


# ------------------------------------------------------------------ permute
def _permute_gpu(x_bits, idx, shard):
    T, k = idx.shape
    H = x_bits.shape[1]
    cap = max(T * k, 1)
    g = Guards()
    x_perm = g.empty((cap, H), torch.bfloat16, fill=0)
    offs = g.empty((shard.n_local_experts + 1,), torch.int32, fill=-5)
    row_src = g.empty((cap,), torch.int32, fill=-5)
    slot_row = g.empty((cap,), torch.int32, fill=-5)
    ws = g.empty(max(B.moe_workspace_bytes(T, k, shard), 1), torch.uint8)
    x_dev = bf16_tensor(x_bits) if T else torch.zeros((1, H), dtype=torch.bfloat16, device="cuda")
    idx_dev = _dev(idx) if T else torch.zeros((1, k), dtype=torch.int32, device="cuda")
    B.moe_permute(x_dev, idx_dev, T, k, shard, x_perm, offs, row_src, slot_row, ws)
    g.check()
    return offs.cpu().numpy(), row_src.cpu().numpy(), slot_row.cpu().numpy(), bf16_bits(x_perm)


@pytest.mark.parametrize("T,k,E,n_local,off", [
    (64, 2, 8, 8, 0), (1500, 2, 8, 8, 0), (1500, 2, 8, 2, 6), (4096, 4, 60, 60, 0), (777, 4, 60, 15, 30),
    (1, 1, 8, 8, 0), (513, 3, 200, 200, 0), (8192, 2, 8, 2, 0), (0, 2, 8, 8, 0), (16, 2, 8, 1, 7),
    (300, 16, 256, 256, 0), (300, 16, 256, 64, 128)])   # E = 256 and k = 16: the limits of the implementation
def test_permute_bit_exact(T, k, E, n_local, off):
    rng = np.random.default_rng(T + k + E)
    H = 64
    x = I.make_x(0, T, H)
    pop = I.zipf_popularity(E)
    idx = np.stack([rng.choice(E, size=k, replace=False, p=pop) for _ in range(T)]).astype(np.int32) \
        if T else np.zeros((0, k), np.int32)
    shard = B.make_shard(E, n_local, off, H, 128, 128)
    offs, row_src, slot_row, x_perm = _permute_gpu(x, idx, shard)
    roffs, rrow_src, rslot_row, rx_perm = O.permute(x, idx, n_local, off)
    R = int(roffs[-1])
    assert np.array_equal(offs, roffs)
    assert np.array_equal(row_src[:R], rrow_src)
    assert np.array_equal(slot_row[:T * k], rslot_row)
    assert np.array_equal(x_perm[:R], rx_perm)
    assert np.all(row_src[R:] == -5)  # nothing written past R


@pytest.mark.parametrize("T,k,E,n_local,off", [
    (16, 2, 8, 8, 0), (32, 2, 8, 8, 0), (16, 4, 60, 60, 0), (16, 4, 60, 15, 30), (8, 8, 64, 64, 0), (4, 16, 256, 256, 0),
    (4, 16, 256, 64, 128), (1, 1, 8, 8, 0), (33, 2, 8, 8, 0), (21, 3, 200, 200, 0), (30, 2, 8, 1, 7), (64, 1, 130, 130, 0)])
def test_permute_index_arrays_alone(T, k, E, n_local, off):
    """x_perm = NULL: only the index arrays are written."""
    rng = np.random.default_rng(7 * T + k + E)
    x = I.make_x(0, T, 64)
    pop = I.zipf_popularity(E)
    idx = np.stack([rng.choice(E, size=k, replace=False, p=pop) for _ in range(T)]).astype(np.int32)
    shard = B.make_shard(E, n_local, off, 64, 128, 128)
    cap = T * k
    offs = torch.full((n_local + 1,), -5, dtype=torch.int32, device="cuda")
    row_src = torch.full((cap,), -5, dtype=torch.int32, device="cuda")
    slot_row = torch.full((cap,), -5, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(B.moe_workspace_bytes(T, k, shard), 1), dtype=torch.uint8, device="cuda")
    B.moe_permute(None, _dev(idx), T, k, shard, None, offs, row_src, slot_row, ws)
    torch.cuda.synchronize()
    roffs, rrow_src, rslot_row, _ = O.permute(x, idx, n_local, off)
    R = int(roffs[-1])
    assert np.array_equal(offs.cpu().numpy(), roffs)
    assert np.array_equal(row_src.cpu().numpy()[:R], rrow_src[:R])
    assert np.all(row_src.cpu().numpy()[R:] == -5)          # entries past R are not touched
    assert np.array_equal(slot_row.cpu().numpy(), rslot_row)


def test_permute_is_deterministic():
    rng = np.random.default_rng(9)
    T, k, E, H = 3000, 4, 60, 64
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    x = I.make_x(0, T, H)
    shard = B.make_shard(E, E, 0, H, 128, 128)
    first = _permute_gpu(x, idx, shard)
    for _ in range(3):
        again = _permute_gpu(x, idx, shard)
        assert all(np.array_equal(a, b) for a, b in zip(first, again))


# ------------------------------------------------------------------ expert FFN
def _ffn_gpu(x_perm_bits, offs, shard, wg, wu, wd, y_bf16=False, gather=None, flags=0):
    """gather = (x_bits [T,H], row_src [cap], k): run moe_expert_ffn_gather on x instead of the permuted copy."""
    cap = x_perm_bits.shape[0]
    g = Guards()
    h_ws = g.empty((cap, shard.inter_slice), torch.bfloat16)
    y = g.empty((cap, shard.hidden), torch.bfloat16 if y_bf16 else torch.float32, fill=float("nan"))
    ws = g.empty(max(B.moe_ffn_workspace_bytes(cap, shard), 16), torch.uint8)
    if gather is not None:
        x_bits, row_src, k = gather
        B.moe_expert_ffn_gather(bf16_tensor(x_bits), _dev(row_src), k, _dev(offs), cap, shard, bf16_tensor(wg),
                                bf16_tensor(wu), bf16_tensor(wd), h_ws, y, ws,
                                flags | (B.MOE_Y_PERM_BF16 if y_bf16 else 0))
    else:
        B.moe_expert_ffn(bf16_tensor(x_perm_bits), _dev(offs), cap, shard, bf16_tensor(wg), bf16_tensor(wu),
                         bf16_tensor(wd), h_ws, y, ws, flags | (B.MOE_Y_PERM_BF16 if y_bf16 else 0))
    g.check()
    return y.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("H,I_s,counts", [
    (512, 1024, [16, 16, 16, 16, 16, 16, 16, 16]),
    (320, 448, [75, 0, 130, 1, 257, 33, 0, 64]),     # ragged rows, empty experts, ragged column tiles
    (64, 64, [5]),
    (256, 192, [300, 129]),
    (2048, 704, [3, 0, 9, 1]),
    (320, 448, [700, 0, 300, 257, 1]),               # large groups: the 256x256 LDS-DMA kernel, ragged everywhere
    (512, 1024, [256, 512]),                         # exact multiples of the tile
    (4096, 3584, [2, 0, 5, 1]),                      # decode: register-resident activations, 8x16 / 8x14 splits
    (4096, 14336, [3, 1]),                           # decode: down projection in 4 K slices + slice sum
    (2048, 1408, [1, 0, 4, 0, 2, 16]),               # decode: 8x8 and 4x11 splits
    (2048, 5632, [12]),                              # shared-expert shape at decode, 2 K slices
    (512, 1024, [16, 2, 0, 9]),                      # decode: generic streaming (H) + 4x8 split (I)
    (512, 1024, [40, 30, 7]),                        # decode regime with more than 32 rows in one expert
    (64, 64, [300, 129, 40]),                        # prefill kernel with a single k-tile (shorter than its pipeline)
    (128, 192, [257, 40, 100]),                      # two and three k-tiles: every tail path of the DMA pipeline
    (192, 128, [100, 500, 64]),
    (256, 320, [64, 128, 21, 256]),                  # four and five k-tiles, all three tile heights
    (512, 4096, [2000]),                             # one expert, few column blocks, long K: down projection in 8 K slices
    (256, 2048, [700, 0, 900]),                      # ... in 4 K slices, with remainder tiles and an empty expert
    # 129 to 192 rows per expert, 128 tiles, K = 48 k-tiles: the sliced down projection pads them to 256-row tiles
    (1024, 3072, [130, 192, 150, 129, 0, 64, 191, 140, 160, 131, 170, 5, 188, 145, 133, 177, 190, 139]),
])
def test_expert_ffn_against_oracle(H, I_s, counts):
    n = len(counts)
    wg, wu, wd = I.make_expert_weights(0, I.MoEShape("f", H, n, 1, I_s, True))
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offs[-1])
    cap = R + 7  # capacity rows beyond R exist and must stay untouched
    xp = I.make_x(1, cap, H)
    shard = B.make_shard(n, n, 0, H, I_s, I_s)
    y = _ffn_gpu(xp, offs, shard, wg, wu, wd)
    ref = O.expert_ffn(xp[:R], offs, wg, wu, wd)
    assert np.all(np.isnan(y[R:])), "rows past R must not be written"
    assert _rel(y[:R], ref) < REL_L2
    assert np.abs(y[:R] - ref).max() < MAX_ABS
    yb = _ffn_gpu(xp, offs, shard, wg, wu, wd, y_bf16=True)
    assert _rel(yb[:R], ref) < REL_L2


@pytest.mark.parametrize("H,I_s,lo,hi,gather", [
    (1024, 192, 226, 330, False),    # 64 experts, a few hundred rows each: one to three 160-row blocks per expert
    (1024, 320, 100, 480, True),     # wide spread around the same average, rows read through row_src
    (2048, 128, 0, 560, False),      # empty experts and experts with four blocks
])
def test_expert_ffn_even_row_blocks(H, I_s, lo, hi, gather):
    """Calls with a few hundred rows per expert run on the tiling with row blocks of 160 rows."""
    n = 64
    rng = np.random.default_rng(H + I_s)
    counts = rng.integers(lo, hi + 1, n)
    counts[5] = 160       # exactly one block
    counts[6] = 161       # one row into the second
    counts[7] = 320
    counts = counts * (270 * n) // int(counts.sum())   # average of 270 rows whatever the spread
    counts[5], counts[6], counts[7] = 160, 161, 320
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offs[-1])
    cap = R + 3
    shard = B.make_shard(n, n, 0, H, I_s, I_s)
    assert B.moe_debug_tile_rows(cap, shard) == 160
    assert B.moe_debug_ffn_plan(cap, shard)[:2] == (False, False)
    wg, wu, wd = I.make_expert_weights(2, I.MoEShape("f", H, n, 1, I_s, True))
    if gather:
        k = 2
        T = (cap + k - 1) // k
        x = I.make_x(3, T, H)
        row_src = rng.permutation(T * k)[:cap].astype(np.int32)
        xp = x[row_src // k]
        y = _ffn_gpu(xp, offs, shard, wg, wu, wd, gather=(x, row_src, k))
    else:
        xp = I.make_x(3, cap, H)
        y = _ffn_gpu(xp, offs, shard, wg, wu, wd)
    ref = O.expert_ffn(xp[:R], offs, wg, wu, wd)
    assert np.all(np.isnan(y[R:])), "rows past R must not be written"
    assert _rel(y[:R], ref) < REL_L2 and np.abs(y[:R] - ref).max() < MAX_ABS
    yb = _ffn_gpu(xp, offs, shard, wg, wu, wd, y_bf16=True)
    assert np.all(np.isnan(yb[R:])) and _rel(yb[:R], ref) < REL_L2
    # each GEMM alone (operator-level timing flags) gives the same bits as the pair
    h_only = _ffn_gpu(xp, offs, shard, wg, wu, wd, flags=B.MOE_FFN_SKIP_DOWN)
    assert np.all(np.isnan(h_only))   # y_perm untouched


def test_expert_ffn_streaming_kernel_with_experts_that_need_several_row_passes():
    """24 small experts, three of them with 17 to 33 rows: 26 (expert, pass) units over 256
    workgroups do not divide evenly, so the ranges of the streaming kernel cross from one unit into
    the next."""
    H, I_s = 2048, 1408
    counts = [3, 1, 0, 17, 5, 2, 8, 33, 1, 4, 0, 6, 2, 9, 20, 1, 3, 7, 2, 5, 1, 4, 6, 2]
    n = len(counts)
    wg, wu, wd = I.make_expert_weights(3, I.MoEShape("f", H, n, 1, I_s, True))
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offs[-1])
    cap = R + 7
    shard = B.make_shard(n, n, 0, H, I_s, I_s)
    assert B.moe_debug_ffn_plan(cap, shard)[:3] == (True, True, 1)   # streaming kernels, 16 rows per pass
    xp = I.make_x(4, cap, H)
    ref = O.expert_ffn(xp[:R], offs, wg, wu, wd)
    y = _ffn_gpu(xp, offs, shard, wg, wu, wd)
    assert np.all(np.isnan(y[R:]))
    assert _rel(y[:R], ref) < REL_L2 and np.abs(y[:R] - ref).max() < MAX_ABS
    # with a sixteenth of the workgroups left out the ranges fall elsewhere; every sum keeps its order
    yl = _ffn_gpu(xp, offs, shard, wg, wu, wd, flags=B.MOE_FFN_LEAVE_ROOM)
    assert np.array_equal(yl[:R], y[:R]) and np.all(np.isnan(yl[R:]))
    # the same call on the tiled kernels
    yt = _ffn_gpu(xp, offs, shard, wg, wu, wd, flags=B.MOE_FFN_TILED)
    assert np.all(np.isnan(yt[R:]))
    assert _rel(yt[:R], ref) < REL_L2 and np.abs(yt[:R] - ref).max() < MAX_ABS


@pytest.mark.parametrize("H,I_s,counts", [(4096, 3584, [2, 0, 5, 1]), (2048, 5632, [12]), (512, 1024, [16, 2, 0, 9])])
def test_expert_ffn_tiled_flag_on_decode_sized_calls(H, I_s, counts):
    n = len(counts)
    wg, wu, wd = I.make_expert_weights(0, I.MoEShape("f", H, n, 1, I_s, True))
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offs[-1])
    cap = R + 7
    xp = I.make_x(1, cap, H)
    shard = B.make_shard(n, n, 0, H, I_s, I_s)
    assert any(B.moe_debug_ffn_plan(cap, shard)[:2])     # left alone, this call streams
    ref = O.expert_ffn(xp[:R], offs, wg, wu, wd)
    for y_bf16 in (False, True):
        y = _ffn_gpu(xp, offs, shard, wg, wu, wd, y_bf16=y_bf16, flags=B.MOE_FFN_TILED)
        assert np.all(np.isnan(y[R:]))
        assert _rel(y[:R], ref) < REL_L2


@pytest.mark.parametrize("seed", range(24))
def test_expert_ffn_random_shapes(seed):
    # seeded random shards: which kernels run, how rows are cut into tiles and what is cut along K
    # all follow from the shape and the routing, so this walks through the combinations
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 13))
    E = n * int(rng.choice([1, 1, 2, 4]))
    H = 64 * int(rng.integers(1, 17))
    I_s = 64 * int(rng.integers(1, 33))
    kind = seed % 4
    if kind == 0:      # decode-sized
        counts = rng.integers(0, 40, n)
    elif kind == 1:    # around the tile heights
        counts = rng.choice([0, 1, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 300, 520], n)
    elif kind == 2:    # one hot expert
        counts = rng.integers(0, 30, n)
        counts[int(rng.integers(0, n))] = int(rng.integers(300, 1500))
    else:
        counts = rng.multinomial(int(rng.integers(200, 2500)), rng.dirichlet(np.ones(n)))
    counts = [int(c) for c in counts]
    wg, wu, wd = I.make_expert_weights(seed, I.MoEShape("f", H, n, 1, I_s, True))
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offs[-1])
    cap = R + int(rng.integers(0, 2000)) if E > n else R + int(rng.integers(0, 9))
    cap = max(cap, 1)
    xp = I.make_x(seed + 1, cap, H)
    shard = B.make_shard(E, n, 0, H, I_s, I_s)
    gather = None
    if seed % 2:   # the FFN reads rows of x through row_src instead of a permuted copy
        k = int(rng.integers(1, 5))
        T = max(1, (R + k - 1) // k + int(rng.integers(0, 5)))
        x = I.make_x(seed + 2, T, H)
        row_src = np.full(cap, -77777, dtype=np.int32)          # entries past R are never to be read
        row_src[:R] = rng.permutation(T * k)[:R] if R <= T * k else rng.integers(0, T * k, R)
        xp = np.zeros_like(xp)
        xp[:R] = x[row_src[:R] // k]
        gather = (x, row_src, k)
    y = _ffn_gpu(xp, offs, shard, wg, wu, wd, gather=gather)
    assert np.all(np.isnan(y[R:])), "rows past R must not be written"
    if R:
        ref = O.expert_ffn(xp[:R], offs, wg, wu, wd)
        assert _rel(y[:R], ref) < REL_L2, (n, E, H, I_s, counts, cap)
        assert np.abs(y[:R] - ref).max() < MAX_ABS, (n, E, H, I_s, counts, cap)


@pytest.mark.parametrize("H,I_s,counts,E,slices", [
    # slices = (256-row blocks whose tiles run whole, K slices of every other tile)
    (512, 4096, [300, 10], 8, (0, 8)),          # 3 row blocks x 2 column blocks: every tile in 8 K slices
    (512, 4096, [3000, 2500], 8, (0, 5)),       # 23 x 2 tiles, 64 k-tiles in 5 uneven slices
    (1024, 4096, [0, 4200], 8, (0, 3)),         # 17 x 4 tiles, the first expert empty
    (2048, 1024, [2500, 2100], 8, (18, 2)),     # 144 tiles run whole, the 8 remainder tiles in 2 slices
    (512, 4096, [0, 0], 8, (0, 1)),
    (2048, 2048, [1300, 40, 800, 2600, 513], 5, (20, 4)),   # 160 tiles whole, 5 x 8 remainder tiles in 4 slices
    (2048, 2048, [1280, 0, 768, 2560, 512], 5, (20, 1)),    # no remainder tiles, 160 of 256 in the last round: nothing is cut
    (2048, 1024, [2048, 1536, 1024, 2304, 1792], 5, (32, 2)),   # 272 tiles: the 16 of the last two row blocks in 2 slices
    (2048, 2048, [2100, 1536, 1024, 2304, 2000], 5, (32, 4)),   # 280 tiles: last three row blocks (one ragged) + remainder tiles
])
def test_expert_ffn_down_projection_cut_along_k_as_the_routing_asks(H, I_s, counts, E, slices):
    # how far the down projection is cut along K follows the routing, not the capacity: a shard
    # that received far fewer rows than its capacity, and the remainder tiles of a large launch
    n = len(counts)
    wg, wu, wd = I.make_expert_weights(0, I.MoEShape("f", H, n, 1, I_s, True))
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(offs[-1])
    cap = 20000 if E > n else R + 9
    xp = I.make_x(1, cap, H)
    shard = B.make_shard(E, n, 0, H, I_s, I_s)
    assert B.moe_debug_ffn_plan(cap, shard)[:2] == (False, False)
    assert B.moe_debug_down_slices(offs, cap, shard)[:2] == slices
    y = _ffn_gpu(xp, offs, shard, wg, wu, wd)
    assert np.all(np.isnan(y[R:])), "rows past R must not be written"
    if R:
        ref = O.expert_ffn(xp[:R], offs, wg, wu, wd)
        assert _rel(y[:R], ref) < REL_L2
        assert np.abs(y[:R] - ref).max() < MAX_ABS


# ------------------------------------------------------------------ combine
@pytest.mark.parametrize("y_bf16,out_f32", [(False, False), (False, True), (True, False)])
@pytest.mark.parametrize("with_shared", [False, True])
def test_combine_against_oracle(y_bf16, out_f32, with_shared):
    rng = np.random.default_rng(4)
    T, k, E, H = 333, 4, 60, 320
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    x = I.make_x(2, T, H)
    _, _, slot_row, _ = O.permute(x, idx, 20, 10)  # an EP shard: many slots are not local
    R = int((slot_row >= 0).sum())
    ydt = torch.bfloat16 if y_bf16 else torch.float32
    y_perm = torch.randn((T * k, H), device="cuda").to(ydt)
    w = rng.random((T, k)).astype(np.float32)
    y_sh = torch.randn((T, H), device="cuda").to(ydt) if with_shared else None
    w_s = I.make_shared_gate_weight(0, H) * 5 if with_shared else None
    out = torch.empty((T, H), dtype=torch.float32 if out_f32 else torch.bfloat16, device="cuda")
    flags = (B.MOE_Y_PERM_BF16 if y_bf16 else 0) | (B.MOE_OUT_F32 if out_f32 else 0)
    B.moe_combine(y_perm, _dev(slot_row), _dev(w), T, k, H, y_sh, bf16_tensor(x) if with_shared else None,
                  _dev(w_s) if with_shared else None, out, flags)
    torch.cuda.synchronize()
    gate = O.shared_gate(x, w_s) if with_shared else None
    ref = O.combine(y_perm.float().cpu().numpy().astype(np.float64), slot_row, w, T, k,
                    y_sh.float().cpu().numpy().astype(np.float64) if with_shared else None, gate)
    got = out.float().cpu().numpy().astype(np.float64)
    if out_f32:
        assert np.abs(got - ref).max() < 1e-5
    else:
        assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-6)  # half a bf16 ulp
    no_local = np.all(slot_row.reshape(T, k) < 0, axis=1)
    if not with_shared:
        assert no_local.any() and np.all(got[no_local] == 0)


# ------------------------------------------------------------------ whole layer, small shapes
def _run_layer(li, **kw):
    layer = ExpertShardLayer.from_inputs(li, **kw)
    g = Guards().wrap_layer(layer)
    x = bf16_tensor(li.x)
    logits = None if li.logits is None else _dev(li.logits)
    y = layer.forward(x, logits).float().cpu().numpy().astype(np.float64)
    g.check()
    return layer, y


def _oracle_layer(li, logits):
    s = li.shape
    shared = (li.ws_gate, li.ws_up, li.ws_down) if li.ws_gate is not None else None
    return O.expert_layer(li.x, logits, s.top_k, s.renorm, s.n_local_experts, s.expert_offset, li.w_gate, li.w_up,
                          li.w_down, shared=shared, w_shared_gate=li.w_shared_gate if shared else None)


def _check_integers(layer, li, T):
    s = li.shape
    logits = layer.logits[:T].cpu().numpy()
    idx, w, _ = O.route_topk(logits, s.top_k, s.renorm)
    assert np.array_equal(layer.topk_idx[:T].cpu().numpy(), idx)
    offs, row_src, slot_row, x_perm = O.permute(li.x, idx, s.n_local_experts, s.expert_offset)
    R = int(offs[-1])
    assert np.array_equal(layer.expert_offsets.cpu().numpy(), offs)
    assert np.array_equal(layer.row_src[:R].cpu().numpy(), row_src)
    assert np.array_equal(layer.slot_row[:T * s.top_k].cpu().numpy(), slot_row)
    if not layer.gathers(T):
        assert np.array_equal(bf16_bits(layer.x_perm[:R]), x_perm)
    return logits


SMALL_TP = I.MoEShape("small-tp", 320, 8, 2, 1792, True, router="uniform")
SMALL_EP = I.MoEShape("small-ep", 320, 8, 2, 448, True, router="zipf")
SMALL_QWEN = I.MoEShape("small-qwen", 256, 60, 4, 192, False, inter_shared=704)


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("out_f32", [False, True])
def test_layer_tiny_config(seed, out_f32):
    li = I.make_layer_inputs(I.TINY, 64, seed)
    layer, y = _run_layer(li, out_f32=out_f32)
    logits = _check_integers(layer, li, 64)
    ref = _oracle_layer(li, logits)
    assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS


def test_layer_tiny_without_renorm():
    li = I.make_layer_inputs(I.MoEShape("tiny-norenorm", 512, 8, 2, 1024, False), 64, 0)
    layer, y = _run_layer(li)
    ref = _oracle_layer(li, _check_integers(layer, li, 64))
    assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS


@pytest.mark.parametrize("tp", [1, 2, 4])
def test_layer_tp_shards_and_partial_sum_invariant(tp):
    T = 300
    full_li = I.make_layer_inputs(SMALL_TP, T, 0)
    logits = None
    acc = np.zeros((T, SMALL_TP.hidden))
    for p in range(tp):
        li = I.make_layer_inputs(SMALL_TP.shard(tp_degree=tp, tp_rank=p), T, 0)
        layer, y = _run_layer(li, out_f32=True)
        logits = _check_integers(layer, li, T)
        ref = _oracle_layer(li, logits)
        assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS
        acc += y
    ref_full = _oracle_layer(full_li, logits)
    assert _rel(acc, ref_full) < 2 * REL_L2 and np.abs(acc - ref_full).max() < 2 * MAX_ABS


@pytest.mark.parametrize("ep", [2, 4, 8])
def test_layer_ep_shards_and_union_invariant(ep):
    T = 700
    full_li = I.make_layer_inputs(SMALL_EP, T, 0)
    acc = np.zeros((T, SMALL_EP.hidden))
    rows = 0
    for q in range(ep):
        li = I.make_layer_inputs(SMALL_EP.shard(ep_degree=ep, ep_rank=q), T, 0)
        layer, y = _run_layer(li, out_f32=True)
        logits = _check_integers(layer, li, T)
        assert np.array_equal(logits, li.logits)
        ref = _oracle_layer(li, logits)
        assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS
        rows += int(layer.expert_offsets[-1].item())
        acc += y
    assert rows == T * 2
    ref_full = _oracle_layer(full_li, full_li.logits)
    assert _rel(acc, ref_full) < 2 * REL_L2 and np.abs(acc - ref_full).max() < 2 * MAX_ABS
    # skewed popularity: the shard holding experts 0.. receives the most rows
    hot = I.make_layer_inputs(SMALL_EP.shard(ep_degree=ep, ep_rank=0), T, 0, weights=False)
    idx, _, _ = O.route_topk(hot.logits, 2, True)
    assert (idx < 8 // ep).sum() > (idx >= 8 - 8 // ep).sum()


@pytest.mark.parametrize("overlap", [True, False])
@pytest.mark.parametrize("T", [32, 96, 500])
def test_layer_qwen_like_with_shared_expert(T, overlap):
    li = I.make_layer_inputs(SMALL_QWEN, T, 0)
    layer, y = _run_layer(li, overlap_shared=overlap)
    ref = _oracle_layer(li, _check_integers(layer, li, T))
    assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS
    # the shared expert may run beside the routed ones on a second stream: repeated calls and
    # replays of a captured graph, with eager work in between, must give the same bits
    x = bf16_tensor(li.x)
    first = layer.forward(x).clone()
    for _ in range(3):
        assert torch.equal(layer.forward(x), first)
    graph, out = layer.capture(x)
    for _ in range(3):
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, first)
        layer.forward(x)
        torch.cuda.synchronize()


@pytest.mark.parametrize("overlap", [True, False])
def test_captured_graph_survives_other_token_counts_and_reallocation(overlap):
    # a graph captured at 16 tokens keeps its own {0, T} offsets and its own buffers: an eager call
    # with more tokens in between, and one that makes the layer allocate larger buffers, must not
    # change what a replay computes
    li16 = I.make_layer_inputs(SMALL_QWEN, 16, 0)
    li48 = I.make_layer_inputs(SMALL_QWEN, 48, 0)    # same seed: same weights, more tokens
    li200 = I.make_layer_inputs(SMALL_QWEN, 200, 0)
    layer = ExpertShardLayer.from_inputs(li16, overlap_shared=overlap, max_tokens=64)
    x16, x48, x200 = bf16_tensor(li16.x), bf16_tensor(li48.x), bf16_tensor(li200.x)
    first = layer.forward(x16).clone()
    graph, out = layer.capture(x16)
    y48 = layer.forward(x48).clone()           # same buffers, other token count
    out.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, first)
    y200 = layer.forward(x200).clone()         # beyond max_tokens: the layer allocates anew
    filler = torch.full((1 << 22,), 1.0, device="cuda")   # anything the allocator hands out now must not be the graph's
    out.zero_()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, first)
    assert torch.equal(layer.forward(x48), y48) and torch.equal(layer.forward(x200), y200)
    ref = _oracle_layer(li200, layer.logits[:200].cpu().numpy())
    assert _rel(y200.float().cpu().numpy().astype(np.float64), ref) < REL_L2
    del filler
    # an explicit stream, shared expert on that same stream
    if not overlap:
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        y = layer.forward(x16, stream=s)
        s.synchronize()
        assert torch.equal(y, first)


def test_layer_hybrid_ep_tp_shard():
    T = 200
    s = SMALL_TP.shard(tp_degree=2, tp_rank=1, ep_degree=2, ep_rank=1)
    li = I.make_layer_inputs(s, T, 0)
    layer, y = _run_layer(li, out_f32=True)
    ref = _oracle_layer(li, _check_integers(layer, li, T))
    assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS


@pytest.mark.parametrize("T", [24, 700])
def test_layer_with_and_without_the_permuted_copy_gives_the_same_bits(T):
    # the FFN either reads x_perm or gathers the same rows of x through row_src: same kernels, same
    # operands, so the layer output must not differ in a single bit
    li = I.make_layer_inputs(SMALL_QWEN, T, 0)
    la, ya = _run_layer(li, gather_in_ffn=True)
    lb, yb = _run_layer(li, gather_in_ffn=False)
    assert la.x_perm is None and lb.x_perm is not None
    assert np.array_equal(ya, yb)
    _check_integers(lb, li, T)


SMALL_ODD = I.MoEShape("small-odd", 256, 12, 4, 1408, False, inter_shared=704)


@pytest.mark.parametrize("tp,T", [(4, 24), (4, 600), (8, 24), (8, 600)])
def test_layer_tp_slices_that_are_not_a_multiple_of_64(tp, T):
    # 1408 / 4 = 352 and 1408 / 8 = 176 (the Qwen1.5-MoE expert size under TP 4 and 8): the layer
    # zero-pads the slice, the partial sums over all ranks still add up to the unsharded layer
    full_li = I.make_layer_inputs(SMALL_ODD, T, 0)
    acc = np.zeros((T, SMALL_ODD.hidden))
    logits = None
    for p in range(tp):
        li = I.make_layer_inputs(SMALL_ODD.shard(tp_degree=tp, tp_rank=p), T, 0)
        assert li.w_gate.shape[1] == 1408 // tp
        layer, y = _run_layer(li, out_f32=True)
        assert layer.ffn_shard.inter_slice % 64 == 0 and layer.shard.inter_slice == 1408 // tp
        logits = _check_integers(layer, li, T)
        ref = _oracle_layer(li, logits)
        assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS
        acc += y
    # every rank adds the gated shared-expert partial sum and its own slice of the routed experts
    ref_full = _oracle_layer(full_li, logits)
    assert _rel(acc, ref_full) < 2 * REL_L2 and np.abs(acc - ref_full).max() < 2 * MAX_ABS


def test_layer_at_the_expert_and_topk_limits():
    s = I.MoEShape("limits", 128, 256, 16, 64, True)
    for T in (7, 130):
        li = I.make_layer_inputs(s, T, 0)
        layer, y = _run_layer(li, out_f32=True)
        ref = _oracle_layer(li, _check_integers(layer, li, T))
        assert _rel(y, ref) < REL_L2 and np.abs(y - ref).max() < MAX_ABS


def test_layer_is_deterministic_and_buffers_reusable():
    li = I.make_layer_inputs(SMALL_QWEN, 500, 0)
    layer = ExpertShardLayer.from_inputs(li)
    x = bf16_tensor(li.x)
    y0 = layer.forward(x).clone()
    y_small = layer.forward(x[:37]).clone()  # smaller batch through the same buffers
    y1 = layer.forward(x).clone()
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    li_small = I.make_layer_inputs(SMALL_QWEN, 37, 0)
    assert np.array_equal(li_small.x, li.x[:37])
    ref = _oracle_layer(li_small, layer.logits[:37].cpu().numpy())  # same rows, same logits as the full batch
    assert _rel(y_small.float().cpu().numpy().astype(np.float64), ref) < REL_L2


def test_graph_replay_matches_eager():
    """A captured layer must give the eager result on every replay, with eager work and
    synchronisations in between (the library records kernels only, never memset nodes)."""
    li = I.make_layer_inputs(SMALL_QWEN, 32, 0)
    layer = ExpertShardLayer.from_inputs(li)
    x = bf16_tensor(li.x)
    eager = layer.forward(x).clone()
    graph, out = layer.capture(x)
    for i in range(4):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), "replay %d differs from eager" % i
        other = layer.forward(bf16_tensor(I.make_x(i + 1, 32, SMALL_QWEN.hidden))).clone()  # eager work in between
        torch.cuda.synchronize()
        assert not torch.equal(other, eager)
    # new contents in the same input buffer are picked up by the next replay
    x2 = bf16_tensor(I.make_x(9, 32, SMALL_QWEN.hidden))
    want = layer.forward(x2).clone()
    x.copy_(x2)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, want)
