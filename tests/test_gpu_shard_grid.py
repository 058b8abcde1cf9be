"""GPU parity over the whole shard grid of the search space: every legal (E_t, E_e) of the three
model shapes (tensor-parallel degree a power of two dividing the expert intermediate size,
expert-parallel degree dividing the expert count, at most 8 devices; the ILP's divisibility
constraints), at a decode-sized and a prefill-sized batch.

For every shard of a configuration: integer outputs in full and the layer output on a stratified
token sample against the oracle.  Over the shards of a configuration: the sum of the shards' fp32
outputs must reproduce the unsharded layer (tensor-parallel partial sums add up, expert-parallel
shard outputs add up).  The shared expert is tensor-parallel sliced and held by the shards of
expert-parallel rank 0 only, so that the sum counts it once."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2508_19373_amd import inputs as I
from paper_2508_19373_amd.latency_table import legal_shards
from paper_2508_19373_amd.layer import ExpertShardLayer, bf16_tensor
from guards import Guards
from sampling import stratified_tokens

pytestmark = pytest.mark.gpu

REL_L2 = 5e-3
MAX_ABS = 2e-2
N_SAMPLE = 512
MODELS = {"mixtral": I.MIXTRAL, "qwen": I.QWEN, "qwen2_57b": I.QWEN2_57B}
TOKENS = (32, 1024)
CASES = [(m, tp, ep, T) for m, base in MODELS.items() for tp, ep in legal_shards(base) for T in TOKENS]

_model = {}


def _load(name):
    """Host and device copies of one model's full weights (one model at a time)."""
    if _model.get("name") != name:
        _model.clear()
        torch.cuda.empty_cache()
        base = MODELS[name]
        li = I.make_layer_inputs(base, 1, 0)
        _model.update(name=name, li=li, full={},
                      dev=tuple(bf16_tensor(w) for w in (li.w_gate, li.w_up, li.w_down)),
                      dev_sh=None if li.ws_gate is None else tuple(bf16_tensor(w) for w in (li.ws_gate, li.ws_up, li.ws_down)),
                      w_router=torch.from_numpy(li.w_router).cuda(),
                      w_sg=None if li.w_shared_gate is None else torch.from_numpy(li.w_shared_gate).cuda())
    return _model


def _slices(m, base, tp, p, ep, q):
    """Shard (p of tp, q of ep) of the weights: device tensors for the layer, host views for the oracle."""
    li = m["li"]
    n_loc, I_s = base.n_experts // ep, base.inter // tp
    es, cs = slice(q * n_loc, (q + 1) * n_loc), slice(p * I_s, (p + 1) * I_s)
    g, u, d = m["dev"]
    dev = (g[es, cs].contiguous(), u[es, cs].contiguous(), d[es, :, cs].contiguous())
    host = O.tp_slice(*O.ep_slice(li.w_gate, li.w_up, li.w_down, ep, q)[:3], tp, p)
    dev_sh = host_sh = None
    if m["dev_sh"] is not None and q == 0:
        s_s = base.inter_shared // tp
        ss = slice(p * s_s, (p + 1) * s_s)
        sg, su, sd = m["dev_sh"]
        dev_sh = (sg[:, ss].contiguous(), su[:, ss].contiguous(), sd[:, :, ss].contiguous())
        host_sh = O.tp_slice(li.ws_gate, li.ws_up, li.ws_down, tp, p)
    return dev, host, dev_sh, host_sh


def _run_shard(m, base, tp, p, ep, q, x, T):
    dev, host, dev_sh, host_sh = _slices(m, base, tp, p, ep, q)
    n_loc = base.n_experts // ep
    layer = ExpertShardLayer(n_experts=base.n_experts, top_k=base.top_k, hidden=base.hidden, inter_full=base.inter,
                             inter_slice=base.inter // tp, n_local_experts=n_loc, expert_offset=q * n_loc,
                             renorm=base.renorm, w_router=m["w_router"], w_gate=dev[0], w_up=dev[1], w_down=dev[2],
                             shared=dev_sh, w_shared_gate=m["w_sg"] if dev_sh is not None else None,
                             inter_shared_full=base.inter_shared, inter_shared_slice=base.inter_shared // tp,
                             max_tokens=T, out_f32=True)
    g = Guards().wrap_layer(layer)
    y = layer.forward(x).cpu().numpy().astype(np.float64)
    g.check()
    return layer, y, host, host_sh


@pytest.mark.parametrize("name,tp,ep,T", CASES)
def test_shard_grid(name, tp, ep, T):
    print("case", name, "tp", tp, "ep", ep, "T", T, flush=True)
    m = _load(name)
    base, li = MODELS[name], m["li"]
    k = base.top_k
    xb = I.make_x(0, T, base.hidden)
    x = bf16_tensor(xb)
    if T not in m["full"]:   # the unsharded layer on the GPU, once per (model, T)
        layer, y, _, _ = _run_shard(m, base, 1, 0, 1, 0, x, T)
        m["full"][T] = (y, layer.logits[:T].cpu().numpy())
        del layer
    y_full, logits = m["full"][T]
    ref_logits = O.router_logits(xb, li.w_router).astype(np.float64)
    assert np.all(np.abs(logits - ref_logits) <= 1e-5 * (1 + np.abs(ref_logits)))
    idx, w32, w64 = O.route_topk(logits, k, base.renorm)

    total, rows_total, worst = np.zeros_like(y_full), 0, (0.0, 0.0)
    for q in range(ep):
        for p in range(tp):
            layer, y, host, host_sh = _run_shard(m, base, tp, p, ep, q, x, T)
            n_loc = base.n_experts // ep
            # every shard routes the whole batch by itself: same logits bit for bit, same decisions
            assert np.array_equal(layer.logits[:T].cpu().numpy(), logits)
            assert np.array_equal(layer.topk_idx[:T].cpu().numpy(), idx)
            assert np.allclose(layer.topk_w[:T].cpu().numpy(), w32, rtol=2e-6, atol=1e-9)
            offs, row_src, slot_row, _ = O.permute(xb, idx, n_loc, q * n_loc)
            R = int(offs[-1])
            assert np.array_equal(layer.expert_offsets.cpu().numpy(), offs)
            assert np.array_equal(layer.row_src[:R].cpu().numpy(), row_src)
            assert np.array_equal(layer.slot_row[:T * k].cpu().numpy(), slot_row)
            if p == 0:
                rows_total += R
            sel, _, _ = stratified_tokens(T, k, offs, row_src, layer.ffn_shard, N_SAMPLE)
            ref = O.expert_layer(xb[sel], None, k, base.renorm, n_loc, q * n_loc, *host, shared=host_sh,
                                 w_shared_gate=li.w_shared_gate if host_sh is not None else None,
                                 topk=(idx[sel], w64[sel]))
            d = y[sel] - ref
            rel, mx = np.linalg.norm(d) / max(np.linalg.norm(ref), 1e-30), np.abs(d).max()
            worst = (max(worst[0], rel), max(worst[1], mx))
            assert rel < REL_L2 and mx < MAX_ABS, (p, q, rel, mx)
            total += y
            del layer
    assert rows_total == T * k   # the expert-parallel shards' rows partition the assignments
    ds = total - y_full
    rel_sum = np.linalg.norm(ds) / np.linalg.norm(y_full)
    print("  %d shards: worst rel-L2 %.3e max-abs %.3e | sum of shards vs unsharded rel-L2 %.3e max-abs %.3e"
          % (tp * ep, worst[0], worst[1], rel_sum, np.abs(ds).max()), flush=True)
    assert rel_sum < 2 * REL_L2 and np.abs(ds).max() < 2 * MAX_ABS
