"""moe_permute_static (the entry point that allocates nothing: its scratch is a static device
array of the library) against moe_permute, through the C ABI: two calls in a row on the same GPU,
the second with a smaller input, both large enough to use the scratch; then the size limit."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2508_19373_amd import binding as B

pytestmark = pytest.mark.gpu


def _run(T, k, E, n_local, off, H, seed, with_copy):
    g = torch.Generator(device="cpu").manual_seed(seed)
    # k distinct experts per token, as a router would select them
    idx = torch.stack([torch.randperm(E, generator=g)[:k] for _ in range(T)]).to(torch.int32).cuda()
    x = torch.randn((T, H), generator=g).to(torch.bfloat16).cuda()
    shard = B.make_shard(E, n_local, off, H, 64, 64)
    cap = T * k

    def bufs():
        return (torch.full((cap, H), -3.0, dtype=torch.bfloat16, device="cuda") if with_copy else None,
                torch.full((n_local + 1,), -7, dtype=torch.int32, device="cuda"),
                torch.full((cap,), -7, dtype=torch.int32, device="cuda"),
                torch.full((cap,), -7, dtype=torch.int32, device="cuda"))
    a, b = bufs(), bufs()
    ws = torch.empty(max(B.moe_workspace_bytes(T, k, shard), 256), dtype=torch.uint8, device="cuda")
    B.moe_permute(x, idx, T, k, shard, a[0], a[1], a[2], a[3], ws)
    B.moe_permute_static(x, idx, T, k, shard, b[0], b[1], b[2], b[3])
    torch.cuda.synchronize()
    assert int(a[1][-1]) > 0
    for u, v in zip(a, b):
        if u is not None:
            assert torch.equal(u.view(torch.int16) if u.dtype == torch.bfloat16 else u, v.view(torch.int16) if v.dtype == torch.bfloat16 else v)
    return int(a[1][-1])


def test_static_permute_equals_permute_on_two_calls_in_a_row():
    print("case static permute: T=5000 k=4 E=60", flush=True)
    assert B.moe_workspace_bytes(5000, 4, B.make_shard(60, 60, 0, 256, 64, 64)) > 256   # uses the scratch
    r1 = _run(5000, 4, 60, 60, 0, 256, 1, True)
    print("case static permute: T=1500 k=2 E=8, experts 2..5 local", flush=True)
    r2 = _run(1500, 2, 8, 4, 2, 128, 2, True)      # smaller input, fewer counts, stale counts behind them
    assert r1 == 20000 and 0 < r2 < 3000
    print("case static permute: T=3000 k=2 E=64, index arrays only", flush=True)
    _run(3000, 2, 64, 64, 0, 64, 3, False)
    print("case static permute: T=64 k=2 E=8 (one-workgroup path, no scratch)", flush=True)
    _run(64, 2, 8, 8, 0, 512, 4, True)


def test_static_permute_rejects_sizes_beyond_its_scratch():
    # ceil(T*k/1024) * n_local > MOE_PERMUTE_STATIC_MAX_COUNTS: refused on the host, nothing enqueued
    E, k = 256, 16
    T = (B.MOE_PERMUTE_STATIC_MAX_COUNTS // E + 1) * 1024 // k
    shard = B.make_shard(E, E, 0, 64, 64, 64)
    assert (T * k + 1023) // 1024 * E > B.MOE_PERMUTE_STATIC_MAX_COUNTS and T * k < (1 << 24)
    P = ctypes.c_void_p(4096)   # never dereferenced: the size check comes first
    st = B.lib().moe_permute_static(None, P, T, k, ctypes.byref(shard), None, P, P, P, None)
    assert st == B.MOE_ERR_WORKSPACE
    # just inside the limit the same arguments pass validation (checked with real buffers)
    T_ok = B.MOE_PERMUTE_STATIC_MAX_COUNTS // E * 1024 // k
    idx = torch.randint(0, E, (T_ok, k), dtype=torch.int32, device="cuda")
    i32 = lambda n: torch.empty(n, dtype=torch.int32, device="cuda")
    offs, rs, sr = i32(E + 1), i32(T_ok * k), i32(T_ok * k)
    B.moe_permute_static(None, idx, T_ok, k, shard, None, offs, rs, sr)
    torch.cuda.synchronize()
    assert int(offs[-1]) == T_ok * k
