"""The C-ABI library loads without a GPU, exports every symbol the header declares, and
rejects invalid arguments on the host before any device call."""
import ctypes
import os
import re

import pytest

from paper_2508_19373_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B._LIB_PATH):
        import __graft_entry__ as g
        g.build()
    return B.lib()


def _declared_functions(header="moe_shard.h"):
    src = open(os.path.join(ROOT, "include", header)).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_every_declared_debug_symbol_is_exported(lib):
    names = _declared_functions("moe_shard_debug.h")
    assert set(names) == set(B.DEBUG_EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    src = open(os.path.join(ROOT, "include", "moe_shard_debug.h")).read()
    assert int(re.search(r"MOE_DEBUG_UNIT_INTS\s+(\d+)", src).group(1)) == B.DEBUG_UNIT_INTS


def test_every_declared_int4_symbol_is_exported_and_validates(lib):
    names = _declared_functions("moe_int4.h")
    assert set(names) == set(B.INT4_EXPORTS)
    src = open(os.path.join(ROOT, "include", "moe_int4.h")).read()
    assert int(re.search(r"MOE_INT4_GROUP\s+(\d+)", src).group(1)) == B.INT4_GROUP
    P = 0x1000
    dq, q = lib.moe_int4_dequantize, lib.moe_int4_quantize
    assert dq(P, P, 100, P, None) == B.MOE_ERR_INVALID_ARG      # not a multiple of the group size
    assert dq(P, P, -64, P, None) == B.MOE_ERR_INVALID_ARG
    assert dq(None, P, 64, P, None) == B.MOE_ERR_INVALID_ARG
    assert dq(P, P, 64, P + 8, None) == B.MOE_ERR_INVALID_ARG   # misaligned
    assert dq(P, P, 0, P, None) == B.MOE_OK                     # empty: nothing launched
    assert q(P, 96, P, P, None) == B.MOE_ERR_INVALID_ARG
    assert q(P, 64, None, P, None) == B.MOE_ERR_INVALID_ARG
    assert q(P, 0, P, P, None) == B.MOE_OK


def test_header_constants_match_binding():
    src = open(os.path.join(ROOT, "include", "moe_shard.h")).read()
    for name in ("MOE_ERR_INVALID_ARG", "MOE_ERR_UNSUPPORTED_SHAPE", "MOE_ERR_WORKSPACE", "MOE_ERR_HIP"):
        m = re.search(name + r"\s*=\s*(-?\d+)", src)
        assert int(m.group(1)) == getattr(B, name)
    for name in ("MOE_RENORM_TOPK", "MOE_LOGITS_GIVEN", "MOE_Y_PERM_BF16", "MOE_OUT_F32", "MOE_FFN_SKIP_GATEUP",
                 "MOE_FFN_SKIP_DOWN", "MOE_FFN_TILED", "MOE_FFN_LEAVE_ROOM"):
        m = re.search(name + r"\s*=\s*1u\s*<<\s*(\d+)", src)
        assert 1 << int(m.group(1)) == getattr(B, name)
    assert ctypes.sizeof(B.MoeShard) == 24


def test_status_strings(lib):
    assert B.status_string(0) == "ok"
    for s in (-1, -2, -3, -4):
        assert B.status_string(s) not in ("ok", "unknown status")
    assert B.status_string(-99) == "unknown status"


P = 0x1000  # a fake, aligned, non-null "device pointer": validation must fail before it is touched


def test_route_topk_validation(lib):
    f = lib.moe_route_topk
    assert f(P, P, P, 4, 64, 8, 0, 0, P, P, None) == B.MOE_ERR_INVALID_ARG       # k < 1
    assert f(P, P, P, 4, 64, 8, 9, 0, P, P, None) == B.MOE_ERR_INVALID_ARG       # k > E
    assert f(P, P, P, 4, 64, 300, 2, 0, P, P, None) == B.MOE_ERR_INVALID_ARG     # E too large
    assert f(P, P, P, -1, 64, 8, 2, 0, P, P, None) == B.MOE_ERR_INVALID_ARG      # T < 0
    assert f(None, P, P, 4, 64, 8, 2, 0, P, P, None) == B.MOE_ERR_INVALID_ARG    # x missing
    assert f(P, P, None, 4, 64, 8, 2, 0, P, P, None) == B.MOE_ERR_INVALID_ARG    # logits missing
    assert f(P, P, P, 4, 60, 8, 2, 0, P, P, None) == B.MOE_ERR_UNSUPPORTED_SHAPE  # H % 8
    assert f(P, P, P, 4, 64, 8, 2, 1 << 7, P, P, None) == B.MOE_ERR_INVALID_ARG  # unknown flag
    assert f(P + 2, P, P, 4, 64, 8, 2, 0, P, P, None) == B.MOE_ERR_INVALID_ARG   # misaligned x


def _shard(**kw):
    d = dict(n_experts=8, n_local_experts=8, expert_offset=0, hidden=512, inter_full=1024, inter_slice=1024)
    d.update(kw)
    return B.MoeShard(**d)


@pytest.mark.parametrize("bad", [
    dict(n_local_experts=0), dict(n_local_experts=3), dict(expert_offset=-1),
    dict(n_local_experts=4, expert_offset=6), dict(inter_slice=300), dict(inter_slice=2048),
    dict(n_experts=0), dict(n_experts=512, n_local_experts=512), dict(hidden=0),
])
def test_shard_descriptor_validation(lib, bad):
    s = _shard(**bad)
    assert B.moe_workspace_bytes(4, 2, s) == 0
    assert lib.moe_permute(P, P, 4, 2, ctypes.byref(s), P, P, P, P, P, 1024, None) == B.MOE_ERR_INVALID_ARG
    assert lib.moe_expert_ffn(P, P, 8, ctypes.byref(s), P, P, P, P, P, P, 1 << 30, 0, None) == B.MOE_ERR_INVALID_ARG


def test_permute_validation(lib):
    s = _shard()
    need = B.moe_workspace_bytes(4, 2, s)
    assert need > 0
    f = lib.moe_permute
    assert f(P, P, 4, 2, None, P, P, P, P, P, need, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 4, 2, ctypes.byref(s), P, P, P, P, P, need - 1, None) == B.MOE_ERR_WORKSPACE
    assert f(P, P, 4, 2, ctypes.byref(s), P, P, P, P, None, need, None) == B.MOE_ERR_WORKSPACE
    assert f(P, None, 4, 2, ctypes.byref(s), P, P, P, P, P, need, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 4, 17, ctypes.byref(s), P, P, P, P, P, need, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 1 << 23, 2, ctypes.byref(s), P, P, P, P, P, need, None) == B.MOE_ERR_INVALID_ARG
    s2 = _shard(hidden=12)
    assert f(P, P, 4, 2, ctypes.byref(s2), P, P, P, P, P, need, None) == B.MOE_ERR_UNSUPPORTED_SHAPE
    # a permuted copy needs x; without one (index arrays only) x may be missing too
    assert f(None, P, 4, 2, ctypes.byref(s), P, P, P, P, P, need, None) == B.MOE_ERR_INVALID_ARG
    assert f(None, P, 4, 2, ctypes.byref(s), None, P, None, P, P, need, None) == B.MOE_ERR_INVALID_ARG   # row_src missing


def test_expert_ffn_validation(lib):
    f = lib.moe_expert_ffn
    s = _shard()
    W = 1 << 30
    assert f(P, P, -1, ctypes.byref(s), P, P, P, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 8, ctypes.byref(s), P, None, P, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 8, ctypes.byref(s), P, P, P, P, P, P, W, B.MOE_OUT_F32, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 8, ctypes.byref(_shard(hidden=520)), P, P, P, P, P, P, W, 0, None) == B.MOE_ERR_UNSUPPORTED_SHAPE
    assert f(P, P, 8, ctypes.byref(_shard(inter_full=1000, inter_slice=500)), P, P, P, P, P, P, W, 0, None) \
        == B.MOE_ERR_UNSUPPORTED_SHAPE
    assert f(P, P, 8, ctypes.byref(s), P, P, P + 8, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG
    # the scheduling hints are accepted (an empty call: nothing is launched), unknown bits are not
    hints = B.MOE_FFN_TILED | B.MOE_FFN_LEAVE_ROOM
    assert f(P, P, 0, ctypes.byref(s), P, P, P, P, P, P, W, hints, None) == B.MOE_OK
    assert f(P, P, 0, ctypes.byref(s), P, P, P, P, P, P, W, 1 << 8, None) == B.MOE_ERR_INVALID_ARG
    # decode-sized call on a Mixtral-shaped shard needs split-K scratch; a prefill-sized one room for the
    # partial sums of tiles cut along K (65536 / 16 column blocks rows, whatever the capacity)
    mix = _shard(hidden=4096, inter_full=14336, inter_slice=14336)
    need = B.moe_ffn_workspace_bytes(32, mix)
    # streaming kernel: 16 wavefronts x 14 k-steps x 2 K slices of 32 rows; the tiled kernels, which
    # MOE_FFN_TILED may ask for, up to 15 further slices of the 32 rows: the larger of the two
    assert need == max(2 * 32 * 4096 * 4, 15 * 32 * 4096 * 4)
    assert B.moe_ffn_workspace_bytes(8192, mix) == 4096 * 4096 * 4
    assert B.moe_ffn_workspace_bytes(8192, _shard(hidden=4096, inter_full=512, inter_slice=512)) == 0   # K too short to cut
    # a single expert with a few hundred rows: the tiled down projection is cut along K
    one = _shard(n_experts=1, n_local_experts=1, hidden=3584, inter_full=20480, inter_slice=20480)
    assert B.moe_ffn_workspace_bytes(1024, one) == (65536 // 14) * 3584 * 4   # up to 16 slices, all but the first in scratch
    assert f(P, P, 32, ctypes.byref(mix), P, P, P, P, P, None, 0, 0, None) == B.MOE_ERR_WORKSPACE
    assert f(P, P, 32, ctypes.byref(mix), P, P, P, P, P, P, need - 1, 0, None) == B.MOE_ERR_WORKSPACE


def test_expert_ffn_gather_validation(lib):
    f = lib.moe_expert_ffn_gather
    s = _shard()
    W = 1 << 30
    assert f(P, None, 2, P, 8, ctypes.byref(s), P, P, P, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG    # no row map
    assert f(P, P, 0, P, 8, ctypes.byref(s), P, P, P, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 17, P, 8, ctypes.byref(s), P, P, P, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG
    assert f(None, P, 2, P, 8, ctypes.byref(s), P, P, P, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, 2, P, -1, ctypes.byref(s), P, P, P, P, P, P, W, 0, None) == B.MOE_ERR_INVALID_ARG
    mix = _shard(hidden=4096, inter_full=14336, inter_slice=14336)
    assert f(P, P, 2, P, 32, ctypes.byref(mix), P, P, P, P, P, None, 0, 0, None) == B.MOE_ERR_WORKSPACE


def test_combine_validation(lib):
    f = lib.moe_combine
    assert f(P, P, P, 4, 2, 512, None, None, None, None, 0, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, P, 4, 2, 512, P, P, None, P, 0, None) == B.MOE_ERR_INVALID_ARG   # x without w_s
    assert f(P, P, P, 4, 2, 512, None, P, P, P, 0, None) == B.MOE_ERR_INVALID_ARG   # gate without y_shared
    assert f(P, P, P, 4, 2, 510, None, None, None, P, 0, None) == B.MOE_ERR_UNSUPPORTED_SHAPE
    assert f(P, P, P, 4, 0, 512, None, None, None, P, 0, None) == B.MOE_ERR_INVALID_ARG
    assert f(P, P, P, 4, 2, 512, None, None, None, P, B.MOE_RENORM_TOPK, None) == B.MOE_ERR_INVALID_ARG


def test_binding_refuses_host_tensors(lib):
    import torch
    t = torch.zeros(4, 8)
    with pytest.raises(ValueError):
        B.moe_route_topk(t, t, t, 4, 8, 8, 2, 0, t, t, stream=0)


def test_public_headers_are_plain_c(tmp_path):
    """The boundary is a C ABI: every header under include/ compiles as C99 on its own."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    inc = os.path.join(ROOT, "include")
    for name in sorted(os.listdir(inc)):
        if not name.endswith(".h"):
            continue
        src = tmp_path / (name + ".c")
        src.write_text('#include "%s"\nint main(void) { return 0; }\n' % name)
        r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-c", str(src),
                            "-o", str(tmp_path / (name + ".o"))], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
