"""One Expert-module call on one shard: owns the device buffers (allocated once through torch)
and issues the C-ABI calls in order.  No arithmetic happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def bf16_tensor(bits: np.ndarray, device="cuda") -> torch.Tensor:
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on the device, same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


FFN_ALIGN = 64  # moe_expert_ffn needs I_s % 64 == 0


def _pad_inter(w_gate, w_up, w_down, inter_slice):
    """Zero-pad an intermediate slice to the next multiple of FFN_ALIGN: extra gate/up rows and
    down columns of zeros add silu(0) * 0 = 0 times 0 to every output, so results are unchanged
    (memory plumbing for tensor-parallel slices such as 1408 / 4 = 352; no arithmetic here)."""
    pad = -inter_slice % FFN_ALIGN
    if pad == 0:
        return w_gate, w_up, w_down, inter_slice
    E, _, H = w_gate.shape
    g = torch.zeros((E, inter_slice + pad, H), dtype=w_gate.dtype, device=w_gate.device)
    u = torch.zeros_like(g)
    d = torch.zeros((E, H, inter_slice + pad), dtype=w_down.dtype, device=w_down.device)
    g[:, :inter_slice].copy_(w_gate)
    u[:, :inter_slice].copy_(w_up)
    d[:, :, :inter_slice].copy_(w_down)
    return g, u, d, inter_slice + pad


_SIDE_STREAMS = {}


def _side_stream(device):
    """One second stream per device for every layer of the process (layers run one after the other)."""
    key = str(torch.device(device))
    if key not in _SIDE_STREAMS:
        _SIDE_STREAMS[key] = torch.cuda.Stream(device=device)
    return _SIDE_STREAMS[key]


def routed_hint_beside_shared(ffn_shard, shared_shard, T) -> int:
    """Scheduling hint (a moe_expert_ffn flag, or 0) for the routed experts' call when the shared
    expert of T tokens runs beside it on a second stream.

    A tiled shared expert cannot start beside resident weight-streaming workgroups (each tiled
    workgroup needs a compute unit's whole LDS): the routed experts are kept tiled too, so that the
    two streams interleave tile by tile.  Measured: -8 to -20 % at 64 to 256 tokens on shards with
    60 or 64 local experts (two or more rounds of tiles even with a few rows per expert, so the
    tiled kernels stream as fast as the streaming kernel); +5 to +16 % on shards with 15 or 30
    experts, hence the tile count.  Those leave 16 compute units to the shared expert instead (30
    experts, 96 / 128 tokens: 177 / 179 -> 170 / 173 us).  A streaming shared expert needs neither."""
    if all(B.moe_debug_ffn_plan(T, shared_shard)[:2]):
        return 0
    gateup_tiles = ffn_shard.n_local_experts * ((ffn_shard.inter_slice + 127) // 128)
    return B.MOE_FFN_TILED if gateup_tiles >= 512 else B.MOE_FFN_LEAVE_ROOM


class ExpertShardLayer:
    """route -> permute -> expert FFN (-> shared expert FFN) -> combine, on the current stream.

    Weights are torch.bfloat16 CUDA tensors in the layouts of include/moe_shard.h.  A slice of
    the intermediate dimension that is not a multiple of 64 is zero-padded once, here, and the
    FFN calls then describe the padded matrices.
    ``y_perm_bf16`` / ``out_f32`` select the element types of the intermediate and the output.
    """

    def __init__(self, *, n_experts, top_k, hidden, inter_full, inter_slice, n_local_experts=None, expert_offset=0,
                 renorm=True, w_router=None, w_gate=None, w_up=None, w_down=None, shared=None, w_shared_gate=None,
                 inter_shared_full=0, inter_shared_slice=0, max_tokens=0, y_perm_bf16=False, out_f32=False,
                 overlap_shared=True, gather_in_ffn=None, device="cuda"):
        n_local_experts = n_experts if n_local_experts is None else n_local_experts
        self.E, self.k, self.H = n_experts, top_k, hidden
        self.shard = B.make_shard(n_experts, n_local_experts, expert_offset, hidden, inter_full, inter_slice)
        self.renorm = renorm
        w_gate, w_up, w_down, padded = _pad_inter(w_gate, w_up, w_down, inter_slice)
        self.ffn_shard = B.make_shard(n_experts, n_local_experts, expert_offset, hidden,
                                      padded * (inter_full // inter_slice), padded)
        self.w_router, self.w_gate, self.w_up, self.w_down = w_router, w_gate, w_up, w_down
        self.w_shared_gate = w_shared_gate
        self.shared, self.shared_shard = None, None
        if shared is not None:
            *self.shared, padded = _pad_inter(*shared, inter_shared_slice)
            self.shared_shard = B.make_shard(1, 1, 0, hidden, padded * (inter_shared_full // inter_shared_slice),
                                             padded)
        self.y_perm_bf16, self.out_f32 = y_perm_bf16, out_f32
        self.device = device
        # the shared expert depends on x only: it may run on a second stream (default priority) beside
        # routing, permutation and the routed experts, and joins before the combine
        # the routed experts can read their rows of x in place through row_src (no permuted copy of
        # x).  That saves about half of moe_permute's time and costs about 1 % of GEMM1's (scattered
        # rows), so by default it is used unless the slice is wide: measured break-even near
        # I_s = 12000 (Mixtral unsharded, I_s = 14336: permute -14 us, GEMM1 +16 us).  The weight-streaming
        # kernel loads its rows once per workgroup either way, so calls that it serves always gather
        # (gathers(T) below).
        self.gather_in_ffn = (inter_slice < 12288) if gather_in_ffn is None else bool(gather_in_ffn)
        self._gather_auto = gather_in_ffn is None
        self.overlap_shared = bool(overlap_shared) and shared is not None
        self._side = _side_stream(device) if self.overlap_shared else None
        self.Tmax = -1
        # {0, T} for the shared expert's call, one immutable device tensor per token count: a
        # captured graph keeps reading the tensor it was captured with
        self._sh_offsets = {}
        # buffers a captured graph still points at are kept alive when a larger batch makes the
        # layer allocate anew, so replaying an older graph stays valid (it works on its own buffers)
        self._captured, self._retired = False, []
        if max_tokens:
            self._alloc(max_tokens)

    _BUFFERS = ("logits", "topk_idx", "topk_w", "x_perm", "expert_offsets", "row_src", "slot_row", "h_ws", "y_perm",
                "workspace", "ffn_ws", "y_out", "h_sh", "y_shared", "ffn_ws_sh")

    def _retire(self, names):
        if self._captured:
            self._retired.extend(getattr(self, n) for n in names if getattr(self, n, None) is not None)

    def _alloc(self, T):
        d, k, H, E = self.device, self.k, self.H, self.E
        self._retire(self._BUFFERS)
        cap = max(T * k, 1)
        Tn = max(T, 1)
        ydt = torch.bfloat16 if self.y_perm_bf16 else torch.float32
        self.logits = torch.empty((Tn, E), dtype=torch.float32, device=d)
        self.topk_idx = torch.empty((Tn, k), dtype=torch.int32, device=d)
        self.topk_w = torch.empty((Tn, k), dtype=torch.float32, device=d)
        self.x_perm = None if self.gather_in_ffn else torch.empty((cap, H), dtype=torch.bfloat16, device=d)
        self.expert_offsets = torch.empty(self.shard.n_local_experts + 1, dtype=torch.int32, device=d)
        self.row_src = torch.empty(cap, dtype=torch.int32, device=d)
        self.slot_row = torch.empty(cap, dtype=torch.int32, device=d)
        self.h_ws = torch.empty((cap, self.ffn_shard.inter_slice), dtype=torch.bfloat16, device=d)
        self.y_perm = torch.empty((cap, H), dtype=ydt, device=d)
        self.workspace = torch.empty(max(B.moe_workspace_bytes(T, k, self.shard), 256), dtype=torch.uint8, device=d)
        self.ffn_ws = torch.empty(max(B.moe_ffn_workspace_bytes(cap, self.ffn_shard), 256), dtype=torch.uint8, device=d)
        self.y_out = torch.empty((Tn, H), dtype=torch.float32 if self.out_f32 else torch.bfloat16, device=d)
        if self.shared is not None:
            self.h_sh = torch.empty((Tn, self.shared_shard.inter_slice), dtype=torch.bfloat16, device=d)
            self.y_shared = torch.empty((Tn, H), dtype=ydt, device=d)
            self.ffn_ws_sh = torch.empty(max(B.moe_ffn_workspace_bytes(Tn, self.shared_shard), 256),
                                         dtype=torch.uint8, device=d)
        self.Tmax = T

    def _shared_offsets(self, T):
        """Device tensor {0, T}: written once, on first use of this token count, and complete
        before this returns (whatever stream the kernels then run on)."""
        t = self._sh_offsets.get(T)
        if t is None:
            if torch.cuda.is_current_stream_capturing():
                raise RuntimeError("run one eager forward with this token count before capturing a graph")
            t = torch.tensor([0, T], dtype=torch.int32).to(self.device)
            torch.cuda.current_stream().synchronize()
            self._sh_offsets[T] = t
        return t

    @property
    def sh_offsets(self):
        """The shared expert's offsets for the most recent token count."""
        return self._sh_offsets[self._last_T]

    def gathers(self, T) -> bool:
        """Whether a forward of T tokens reads the routed experts' rows of x in place (no permuted copy)."""
        if self.gather_in_ffn or not self._gather_auto:
            return self.gather_in_ffn
        return bool(B.moe_debug_ffn_plan(T * self.k, self.ffn_shard)[0])   # GEMM1 on the streaming kernel

    def forward(self, x: torch.Tensor, logits: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        T = x.shape[0]
        if T > self.Tmax:
            if torch.cuda.is_current_stream_capturing():
                raise RuntimeError("run one eager forward with this token count before capturing a graph")
            self._alloc(T)
        self._last_T = T
        k, H, E = self.k, self.H, self.E
        # the FFN scratch depends on the regime (decode-sized calls need split-K partials)
        need = B.moe_ffn_workspace_bytes(T * k, self.ffn_shard)
        if need > self.ffn_ws.numel():
            self._retire(("ffn_ws",))
            self.ffn_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        if self.shared is not None:
            need = B.moe_ffn_workspace_bytes(T, self.shared_shard)
            if need > self.ffn_ws_sh.numel():
                self._retire(("ffn_ws_sh",))
                self.ffn_ws_sh = torch.empty(need, dtype=torch.uint8, device=self.device)
        flags = B.MOE_RENORM_TOPK if self.renorm else 0
        if logits is not None:
            self.logits[:T].copy_(logits)
            flags |= B.MOE_LOGITS_GIVEN
        yflag = B.MOE_Y_PERM_BF16 if self.y_perm_bf16 else 0
        rflag = yflag
        if self.shared is not None and self.overlap_shared:
            rflag |= routed_hint_beside_shared(self.ffn_shard, self.shared_shard, T)
        y_shared, joined = None, None
        if self.shared is not None:
            sh_offsets = self._shared_offsets(T)
            y_shared = self.y_shared
        if self.shared is not None and self.overlap_shared:
            if stream is not None:
                raise ValueError("overlap_shared works on torch's current stream only")
            main = torch.cuda.current_stream()
            self._side.wait_stream(main)          # x (and sh_offsets) are ready where main stands now
            # a streaming shared expert leaves 16 compute units free, so that the router and the
            # permutation on the main stream, each a workgroup or two on the critical path, start
            # at once instead of waiting for a resident workgroup to finish (-2 to -3.5 % at 16 to 64 tokens)
            B.moe_expert_ffn(x, sh_offsets, T, self.shared_shard, self.shared[0], self.shared[1], self.shared[2],
                             self.h_sh, self.y_shared, self.ffn_ws_sh, yflag | B.MOE_FFN_LEAVE_ROOM, self._side)
            joined = self._side
        B.moe_route_topk(x, self.w_router, self.logits, T, H, E, k, flags, self.topk_idx, self.topk_w, stream)
        gather = self.gathers(T)
        B.moe_permute(x, self.topk_idx, T, k, self.shard, None if gather else self.x_perm, self.expert_offsets,
                      self.row_src, self.slot_row, self.workspace, stream=stream)
        if gather:
            B.moe_expert_ffn_gather(x, self.row_src, k, self.expert_offsets, T * k, self.ffn_shard, self.w_gate,
                                    self.w_up, self.w_down, self.h_ws, self.y_perm, self.ffn_ws, rflag, stream)
        else:
            B.moe_expert_ffn(self.x_perm, self.expert_offsets, T * k, self.ffn_shard, self.w_gate, self.w_up,
                             self.w_down, self.h_ws, self.y_perm, self.ffn_ws, rflag, stream)
        if self.shared is not None and not self.overlap_shared:
            B.moe_expert_ffn(x, sh_offsets, T, self.shared_shard, self.shared[0], self.shared[1], self.shared[2],
                             self.h_sh, self.y_shared, self.ffn_ws_sh, yflag, stream)
        if joined is not None:
            torch.cuda.current_stream().wait_stream(joined)
        cflags = yflag | (B.MOE_OUT_F32 if self.out_f32 else 0)
        gate_x = x if self.w_shared_gate is not None else None
        B.moe_combine(self.y_perm, self.slot_row, self.topk_w, T, k, H, y_shared, gate_x, self.w_shared_gate,
                      self.y_out, cflags, stream)
        return self.y_out[:T]

    def capture(self, x: torch.Tensor, logits: torch.Tensor | None = None):
        """Capture one forward on (x, logits) into a HIP graph; returns (graph, output view).
        Decode-sized layers are a chain of short kernels, so replaying a graph removes most of
        the launch gaps.  The library enqueues kernels only (no memset nodes, no allocation),
        which is what makes the capture legal; x / logits are read in place at every replay."""
        self.forward(x, logits)  # eager warm-up: sizes the buffers, sets the shared-expert offsets
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        self._captured = True
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                out = self.forward(x, logits)
        torch.cuda.current_stream().wait_stream(side)
        return graph, out

    @classmethod
    def from_inputs(cls, li, **kw) -> "ExpertShardLayer":
        """Build from paper_2508_19373_amd.inputs.LayerInputs (uploads the weights)."""
        s = li.shape
        kw.setdefault("max_tokens", li.T)
        shared = None
        if li.ws_gate is not None:
            shared = tuple(bf16_tensor(w) for w in (li.ws_gate, li.ws_up, li.ws_down))
        return cls(n_experts=s.n_experts, top_k=s.top_k, hidden=s.hidden, inter_full=s.inter,
                   inter_slice=s.inter_slice, n_local_experts=s.n_local_experts, expert_offset=s.expert_offset,
                   renorm=s.renorm,
                   w_router=None if li.w_router is None else torch.from_numpy(li.w_router).cuda(),
                   w_gate=bf16_tensor(li.w_gate), w_up=bf16_tensor(li.w_up), w_down=bf16_tensor(li.w_down),
                   shared=shared,
                   w_shared_gate=None if (li.w_shared_gate is None or shared is None) else torch.from_numpy(li.w_shared_gate).cuda(),
                   inter_shared_full=s.inter_shared, inter_shared_slice=s.inter_shared_slice,
                   **kw)
