"""ctypes binding of libmoe_shard.so: same names as the C ABI (include/moe_shard.h), argument
marshalling only.  Tensors are torch CUDA tensors (PyTorch supplies device memory and the
stream); every step of the path runs in the library's HIP kernels.  There is no fallback: a
missing library raises at first use."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmoe_shard.so")
_lib = None

MOE_OK = 0
MOE_ERR_INVALID_ARG = -1
MOE_ERR_UNSUPPORTED_SHAPE = -2
MOE_ERR_WORKSPACE = -3
MOE_ERR_HIP = -4
MOE_RENORM_TOPK = 1 << 0
MOE_LOGITS_GIVEN = 1 << 1
MOE_Y_PERM_BF16 = 1 << 2
MOE_OUT_F32 = 1 << 3
MOE_FFN_SKIP_GATEUP = 1 << 4
MOE_FFN_SKIP_DOWN = 1 << 5
MOE_FFN_TILED = 1 << 6
MOE_FFN_LEAVE_ROOM = 1 << 7
MOE_MAX_EXPERTS = 256
MOE_MAX_TOPK = 16
MOE_PERMUTE_STATIC_MAX_COUNTS = 262144

EXPORTS = ("moe_route_topk", "moe_permute", "moe_permute_static", "moe_expert_ffn", "moe_expert_ffn_gather", "moe_combine", "moe_workspace_bytes",
           "moe_ffn_workspace_bytes", "moe_status_string")
DEBUG_EXPORTS = ("moe_debug_gemm_units", "moe_debug_ffn_plan", "moe_debug_down_slices", "moe_debug_device_units",
                 "moe_debug_tile_rows", "moe_debug_even_units")
INT4_EXPORTS = ("moe_int4_dequantize", "moe_int4_quantize")
INT4_GROUP = 64
DEBUG_UNIT_INTS = 5
DEBUG_SLICE_INTS = 8
DEBUG_DEVICE_INTS = 9


class MoeShard(ctypes.Structure):
    _fields_ = [("n_experts", ctypes.c_int32), ("n_local_experts", ctypes.c_int32),
                ("expert_offset", ctypes.c_int32), ("hidden", ctypes.c_int32),
                ("inter_full", ctypes.c_int32), ("inter_slice", ctypes.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (fn, status_string(status), status))


def lib() -> ctypes.CDLL:
    """Load the HIP library (built in-tree by __graft_entry__.build()).  No CPU fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libmoe_shard.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, u32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_uint32, ctypes.c_size_t
        shp = ctypes.POINTER(MoeShard)
        L.moe_route_topk.argtypes = [vp, vp, vp, i32, i32, i32, i32, u32, vp, vp, vp]
        L.moe_route_topk.restype = ctypes.c_int
        L.moe_permute.argtypes = [vp, vp, i32, i32, shp, vp, vp, vp, vp, vp, sz, vp]
        L.moe_permute.restype = ctypes.c_int
        L.moe_permute_static.argtypes = [vp, vp, i32, i32, shp, vp, vp, vp, vp, vp]
        L.moe_permute_static.restype = ctypes.c_int
        L.moe_expert_ffn.argtypes = [vp, vp, i32, shp, vp, vp, vp, vp, vp, vp, sz, u32, vp]
        L.moe_expert_ffn.restype = ctypes.c_int
        L.moe_expert_ffn_gather.argtypes = [vp, vp, i32, vp, i32, shp, vp, vp, vp, vp, vp, vp, sz, u32, vp]
        L.moe_expert_ffn_gather.restype = ctypes.c_int
        L.moe_combine.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, u32, vp]
        L.moe_combine.restype = ctypes.c_int
        L.moe_workspace_bytes.argtypes = [i32, i32, shp]
        L.moe_workspace_bytes.restype = sz
        L.moe_ffn_workspace_bytes.argtypes = [i32, shp]
        L.moe_ffn_workspace_bytes.restype = sz
        L.moe_status_string.argtypes = [ctypes.c_int]
        L.moe_status_string.restype = ctypes.c_char_p
        L.moe_int4_dequantize.argtypes = [vp, vp, ctypes.c_int64, vp, vp]
        L.moe_int4_dequantize.restype = ctypes.c_int
        L.moe_int4_quantize.argtypes = [vp, ctypes.c_int64, vp, vp, vp]
        L.moe_int4_quantize.restype = ctypes.c_int
        L.moe_debug_ffn_plan.argtypes = [i32, shp, vp]
        L.moe_debug_ffn_plan.restype = i32
        L.moe_debug_down_slices.argtypes = [vp, i32, shp, vp, vp, i32]
        L.moe_debug_down_slices.restype = i32
        L.moe_debug_device_units.argtypes = [vp, i32, i32, i32, i32, i32, vp, i32, vp]
        L.moe_debug_device_units.restype = i32
        L.moe_debug_gemm_units.argtypes = [vp, i32, i32, i32, vp, i32]
        L.moe_debug_gemm_units.restype = i32
        L.moe_debug_even_units.argtypes = [vp, i32, i32, i32, vp, i32]
        L.moe_debug_even_units.restype = i32
        L.moe_debug_tile_rows.argtypes = [i32, shp]
        L.moe_debug_tile_rows.restype = i32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().moe_status_string(int(status)).decode()


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("device tensor required")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor required")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _check(fn: str, status: int):
    if status != MOE_OK:
        raise MoeError(fn, status)


def make_shard(n_experts, n_local_experts, expert_offset, hidden, inter_full, inter_slice) -> MoeShard:
    return MoeShard(n_experts, n_local_experts, expert_offset, hidden, inter_full, inter_slice)


def moe_route_topk(x, w_router, logits, T, H, E, k, flags, topk_idx, topk_w, stream=None):
    _check("moe_route_topk", lib().moe_route_topk(_ptr(x), _ptr(w_router), _ptr(logits), T, H, E, k, flags,
                                                  _ptr(topk_idx), _ptr(topk_w), _stream(stream)))


def moe_workspace_bytes(T, k, shard: MoeShard) -> int:
    return int(lib().moe_workspace_bytes(T, k, ctypes.byref(shard)))


def moe_permute(x, topk_idx, T, k, shard: MoeShard, x_perm, expert_offsets, row_src, slot_row, workspace,
                workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check("moe_permute", lib().moe_permute(_ptr(x), _ptr(topk_idx), T, k, ctypes.byref(shard), _ptr(x_perm),
                                            _ptr(expert_offsets), _ptr(row_src), _ptr(slot_row), _ptr(workspace),
                                            workspace_bytes, _stream(stream)))


def moe_permute_static(x, topk_idx, T, k, shard: MoeShard, x_perm, expert_offsets, row_src, slot_row, stream=None):
    _check("moe_permute_static", lib().moe_permute_static(_ptr(x), _ptr(topk_idx), T, k, ctypes.byref(shard),
                                                          _ptr(x_perm), _ptr(expert_offsets), _ptr(row_src),
                                                          _ptr(slot_row), _stream(stream)))


def moe_ffn_workspace_bytes(cap_rows, shard: MoeShard) -> int:
    return int(lib().moe_ffn_workspace_bytes(cap_rows, ctypes.byref(shard)))


def moe_expert_ffn(x_perm, expert_offsets, cap_rows, shard: MoeShard, w_gate, w_up, w_down, h_workspace, y_perm,
                   workspace=None, flags=0, stream=None):
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("moe_expert_ffn", lib().moe_expert_ffn(_ptr(x_perm), _ptr(expert_offsets), cap_rows, ctypes.byref(shard),
                                                  _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(h_workspace),
                                                  _ptr(y_perm), _ptr(workspace), wbytes, flags, _stream(stream)))


def moe_expert_ffn_gather(x, row_src, k, expert_offsets, cap_rows, shard: MoeShard, w_gate, w_up, w_down, h_workspace,
                          y_perm, workspace=None, flags=0, stream=None):
    wbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check("moe_expert_ffn_gather",
           lib().moe_expert_ffn_gather(_ptr(x), _ptr(row_src), k, _ptr(expert_offsets), cap_rows, ctypes.byref(shard),
                                       _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(h_workspace), _ptr(y_perm),
                                       _ptr(workspace), wbytes, flags, _stream(stream)))


def moe_combine(y_perm, slot_row, topk_w, T, k, H, y_shared, x, w_shared_gate, y_out, flags=0, stream=None):
    _check("moe_combine", lib().moe_combine(_ptr(y_perm), _ptr(slot_row), _ptr(topk_w), T, k, H, _ptr(y_shared),
                                            _ptr(x), _ptr(w_shared_gate), _ptr(y_out), flags, _stream(stream)))


def moe_int4_dequantize(codes, qparams, n_elems, w_bf16, stream=None):
    _check("moe_int4_dequantize", lib().moe_int4_dequantize(_ptr(codes), _ptr(qparams), n_elems, _ptr(w_bf16),
                                                            _stream(stream)))


def moe_int4_quantize(w_bf16, n_elems, codes, qparams, stream=None):
    _check("moe_int4_quantize", lib().moe_int4_quantize(_ptr(w_bf16), n_elems, _ptr(codes), _ptr(qparams),
                                                        _stream(stream)))


def moe_debug_gemm_units(expert_offsets, cap_rows, n_col_blocks):
    """Host-only: the prefill grouped GEMM's work list for one routing, as an int32 array
    [grid, DEBUG_UNIT_INTS] (see include/moe_shard_debug.h).  `expert_offsets` is a host sequence."""
    import numpy as np
    offs = np.ascontiguousarray(expert_offsets, dtype=np.int32)
    n_local = offs.size - 1
    max_units = 8 * (((cap_rows // 256 + n_local) * n_col_blocks + 7) // 8 + 2 * ((n_local * n_col_blocks + 7) // 8))
    out = np.zeros((max_units, DEBUG_UNIT_INTS), dtype=np.int32)
    n = lib().moe_debug_gemm_units(offs.ctypes.data, n_local, cap_rows, n_col_blocks,
                                   out.ctypes.data, max_units)
    if n < 0:
        raise MoeError("moe_debug_gemm_units", n)
    return out[:n]


def moe_debug_even_units(expert_offsets, cap_rows, n_col_blocks):
    """Host-only: the work list of the 160-row tiling for one routing, records as moe_debug_gemm_units."""
    import numpy as np
    offs = np.ascontiguousarray(expert_offsets, dtype=np.int32)
    n_local = offs.size - 1
    max_units = 8 * (((cap_rows // 160 + n_local) * n_col_blocks + 7) // 8)
    out = np.zeros((max(max_units, 1), DEBUG_UNIT_INTS), dtype=np.int32)
    n = lib().moe_debug_even_units(offs.ctypes.data, n_local, cap_rows, n_col_blocks, out.ctypes.data, max_units)
    if n < 0:
        raise MoeError("moe_debug_even_units", n)
    return out[:n]


def moe_debug_tile_rows(cap_rows, shard: MoeShard) -> int:
    """Host-only: row-block height (256 or 160) of the tiled kernels moe_expert_ffn would use."""
    n = lib().moe_debug_tile_rows(cap_rows, ctypes.byref(shard))
    if n < 0:
        raise MoeError("moe_debug_tile_rows", n)
    return int(n)


def moe_debug_down_slices(expert_offsets, cap_rows, shard: MoeShard, with_units=False):
    """Host-only: how the tiled fp32 down projection is cut along K for this routing (see
    include/moe_shard_debug.h): (slices of the 256-row tiles, slices of the remainder tiles, rows
    with partial sums, scratch rows provided), and with `with_units` also the per-workgroup records
    [grid, DEBUG_SLICE_INTS].  `expert_offsets` is a host sequence."""
    import numpy as np
    offs = np.ascontiguousarray(expert_offsets, dtype=np.int32)
    if offs.size != shard.n_local_experts + 1:
        raise ValueError("expert_offsets must have n_local_experts + 1 entries")
    info = (ctypes.c_int32 * 4)()
    n = lib().moe_debug_down_slices(offs.ctypes.data, cap_rows, ctypes.byref(shard), info, None, 0)
    if n < 0:
        raise MoeError("moe_debug_down_slices", n)
    if not with_units:
        return tuple(info)
    out = np.zeros((n, DEBUG_SLICE_INTS), dtype=np.int32)
    n = lib().moe_debug_down_slices(offs.ctypes.data, cap_rows, ctypes.byref(shard), info, out.ctypes.data, n)
    if n < 0:
        raise MoeError("moe_debug_down_slices", n)
    return tuple(info), out[:n]


def moe_debug_device_units(expert_offsets, cap_rows, n_col_blocks, nk, max_slices, stream=None):
    """The GEMM kernels' own (wave-parallel) evaluation of the work list, run on the device:
    int32 tensor [grid, DEBUG_DEVICE_INTS] (see include/moe_shard_debug.h).  `expert_offsets` is a
    device int32 tensor."""
    import torch
    n_local = expert_offsets.numel() - 1
    max_units = 8 * ((cap_rows // 256 + n_local) * n_col_blocks // 8 + 1 + 2 * (n_local * n_col_blocks // 8 + 1) + 64)
    out = torch.full((max_units, DEBUG_DEVICE_INTS), -7, dtype=torch.int32, device=expert_offsets.device)
    n = lib().moe_debug_device_units(_ptr(expert_offsets), n_local, cap_rows, n_col_blocks, nk, max_slices,
                                     _ptr(out), max_units, _stream(stream))
    if n < 0:
        raise MoeError("moe_debug_device_units", n)
    return out[:n]


def moe_debug_ffn_plan(cap_rows, shard: MoeShard):
    """Host-only: (GEMM1 by the streaming kernel, GEMM2 by the streaming kernel, rows per pass / 16,
    K slices of GEMM2) that moe_expert_ffn would use (see include/moe_shard_debug.h)."""
    plan = (ctypes.c_int32 * 4)()
    st = lib().moe_debug_ffn_plan(cap_rows, ctypes.byref(shard), plan)
    if st != MOE_OK:
        raise MoeError("moe_debug_ffn_plan", st)
    return bool(plan[0]), bool(plan[1]), int(plan[2]), int(plan[3])
