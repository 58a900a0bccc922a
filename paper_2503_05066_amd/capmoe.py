"""Thin binding to libcapmoe.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (PyTorch is used for device memory and streams, nothing
else); every step of the layer runs in the library's HIP kernels.  There is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import math
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcapmoe.so")

MOE_OK = 0
MODE_NONE, MODE_TOKEN_DROP, MODE_EXPANDED_DROP = 0, 1, 2
SCOPE_LOCAL, SCOPE_GLOBAL, SCOPE_LOCAL_DEVICE, SCOPE_GLOBAL_DEVICE = 0, 1, 2, 3
DTYPE_F32, DTYPE_BF16 = 0, 1
METRIC_SCORE, METRIC_ORDER, METRIC_REVERSE_ORDER, METRIC_RANDOM = 0, 1, 2, 3


class MoeDesc(ctypes.Structure):
    """moe_desc_t of include/capmoe.h."""

    _fields_ = [
        ("n_tokens", ctypes.c_int32), ("d_model", ctypes.c_int32), ("n_experts", ctypes.c_int32),
        ("top_k", ctypes.c_int32), ("d_hidden", ctypes.c_int32), ("device_groups", ctypes.c_int32),
        ("mode", ctypes.c_int32), ("capacity_scope", ctypes.c_int32), ("gamma", ctypes.c_double),
        ("dtype", ctypes.c_int32), ("metric", ctypes.c_int32),
        ("overselect", ctypes.c_int32), ("max_experts", ctypes.c_int32),
    ]


KERNELS = ("router_logits", "softmax_topk", "drop_prepare", "drop_select", "drop_emit", "dispatch", "ffn_schedule",
           "ffn_gate_up", "ffn_down", "combine", "drop_limit")


class MoeProfile(ctypes.Structure):
    """moe_profile_t of include/capmoe.h: event handles per kernel id and the library's launch counts."""

    _fields_ = [("start", ctypes.c_void_p * len(KERNELS)), ("stop", ctypes.c_void_p * len(KERNELS)),
                ("launches", ctypes.c_int64 * len(KERNELS))]

    def set_events(self, kernel: int, start_event, stop_event):
        """torch.cuda.Event pair (created with enable_timing) for one kernel id, or None, None."""
        def handle(ev):
            if ev is None:
                return None
            if not ev.cuda_event:      # torch creates the hipEvent lazily; recording once materialises it
                ev.record()
            return ev.cuda_event
        self.start[kernel] = handle(start_event)
        self.stop[kernel] = handle(stop_event)


class CapMoeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} (status {status})")


_lib = None


def load():
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_05066_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        dp = ctypes.POINTER(MoeDesc)
        lib.moe_status_string.argtypes = [i32]
        lib.moe_status_string.restype = ctypes.c_char_p
        lib.moe_query.argtypes = [dp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                                  ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_size_t)]
        lib.moe_route_topk.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_route_topk_static.argtypes = [dp, vp, vp, vp, i32, vp, vp, vp, vp, vp]
        lib.moe_capacity_drop.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_capacity_drop_ranked.argtypes = [dp, vp, vp, vp, ctypes.c_uint32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_dispatch.argtypes = [dp, vp, vp, vp, vp, vp]
        lib.moe_grouped_ffn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_dispatch_ffn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.moe_combine.argtypes = [dp, vp, vp, vp, vp, vp]
        lib.moe_layer_forward.argtypes = [dp] + [vp] * 7 + [ctypes.c_uint32] + [vp] * 13 + [sz, vp]
        lib.moe_layer_forward.restype = i32
        lib.moe_profile_attach.argtypes = [ctypes.POINTER(MoeProfile)]
        lib.moe_profile_attach.restype = i32
        lib.moe_ffn_schedule_query.argtypes = [ctypes.POINTER(MoeDesc), vp, i32, vp, vp]
        lib.moe_ffn_schedule_query.restype = i32
        lib.moe_probe_mfma_bf16.argtypes = [i32, i32, i32, vp, ctypes.POINTER(ctypes.c_int64), vp]
        lib.moe_probe_mfma_bf16.restype = i32
        for f in ("moe_query", "moe_route_topk", "moe_route_topk_static", "moe_capacity_drop", "moe_capacity_drop_ranked", "moe_dispatch",
                  "moe_grouped_ffn",
                  "moe_dispatch_ffn", "moe_combine"):
            getattr(lib, f).restype = i32
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().moe_status_string(int(status)).decode()


def make_desc(n_tokens, d_model, n_experts, top_k, d_hidden, device_groups=1, mode=MODE_TOKEN_DROP,
              capacity_scope=SCOPE_LOCAL, gamma=1.0, dtype=DTYPE_BF16, metric=METRIC_SCORE, overselect=0,
              max_experts=0) -> MoeDesc:
    return MoeDesc(n_tokens, d_model, n_experts, top_k, d_hidden, device_groups, mode, capacity_scope,
                   float(gamma), dtype, metric, overselect, int(max_experts))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch

        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, what: str):
    if status != MOE_OK:
        raise CapMoeError(status, what)


def moe_query(desc: MoeDesc):
    """(cap, slots_per_token, max_rows, workspace_bytes) of a descriptor; host only."""
    cap, slots = ctypes.c_int32(), ctypes.c_int32()
    rows, ws = ctypes.c_int64(), ctypes.c_size_t()
    _check(load().moe_query(ctypes.byref(desc), ctypes.byref(cap), ctypes.byref(slots), ctypes.byref(rows),
                            ctypes.byref(ws)), "moe_query")
    return cap.value, slots.value, rows.value, ws.value


def moe_route_topk(desc, x, w_router, bias, use_given_logits, logits, scores, topk_idx, topk_score, workspace,
                   stream=None):
    _check(load().moe_route_topk(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(bias), int(use_given_logits),
                                 _ptr(logits), _ptr(scores), _ptr(topk_idx), _ptr(topk_score), _ptr(workspace),
                                 workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                 _stream(stream)), "moe_route_topk")


def moe_route_topk_static(desc, x, w_router, bias, use_given_logits, logits, scores, topk_idx, topk_score, stream=None):
    _check(load().moe_route_topk_static(ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(bias),
                                        int(use_given_logits), _ptr(logits), _ptr(scores), _ptr(topk_idx),
                                        _ptr(topk_score), _stream(stream)), "moe_route_topk_static")


def moe_capacity_drop(desc, scores, topk_idx, expert_count, seg_count, expert_offset, row_token, row_weight,
                      pair_row, workspace, stream=None):
    _check(load().moe_capacity_drop(ctypes.byref(desc), _ptr(scores), _ptr(topk_idx), _ptr(expert_count),
                                    _ptr(seg_count), _ptr(expert_offset), _ptr(row_token), _ptr(row_weight),
                                    _ptr(pair_row), _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream(stream)), "moe_capacity_drop")


def moe_capacity_drop_ranked(desc, scores, topk_idx, token_class, seed, expert_count, seg_count, expert_offset,
                             row_token, row_weight, pair_row, workspace, stream=None):
    _check(load().moe_capacity_drop_ranked(ctypes.byref(desc), _ptr(scores), _ptr(topk_idx), _ptr(token_class),
                                           int(seed) & 0xFFFFFFFF, _ptr(expert_count), _ptr(seg_count),
                                           _ptr(expert_offset), _ptr(row_token), _ptr(row_weight), _ptr(pair_row),
                                           _ptr(workspace), workspace.numel() * workspace.element_size(),
                                           _stream(stream)), "moe_capacity_drop_ranked")


def moe_dispatch(desc, x, expert_offset, row_token, xp, stream=None):
    _check(load().moe_dispatch(ctypes.byref(desc), _ptr(x), _ptr(expert_offset), _ptr(row_token), _ptr(xp),
                               _stream(stream)), "moe_dispatch")


def moe_grouped_ffn(desc, xp, expert_offset, w_gate, w_up, w_down, yp, workspace, stream=None):
    _check(load().moe_grouped_ffn(ctypes.byref(desc), _ptr(xp), _ptr(expert_offset), _ptr(w_gate), _ptr(w_up),
                                  _ptr(w_down), _ptr(yp), _ptr(workspace),
                                  workspace.numel() * workspace.element_size(), _stream(stream)), "moe_grouped_ffn")


def moe_dispatch_ffn(desc, x, expert_offset, row_token, w_gate, w_up, w_down, yp, workspace, stream=None):
    _check(load().moe_dispatch_ffn(ctypes.byref(desc), _ptr(x), _ptr(expert_offset), _ptr(row_token), _ptr(w_gate),
                                   _ptr(w_up), _ptr(w_down), _ptr(yp), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream(stream)), "moe_dispatch_ffn")


def moe_combine(desc, yp, row_weight, pair_row, y, stream=None):
    _check(load().moe_combine(ctypes.byref(desc), _ptr(yp), _ptr(row_weight), _ptr(pair_row), _ptr(y),
                              _stream(stream)), "moe_combine")


def moe_layer_forward(desc, x, w_router, bias, w_gate, w_up, w_down, token_class, seed, buf, stream=None):
    """The whole layer through the one-call entry point, into the buffers of a LayerBuffers."""
    ws = buf.workspace
    _check(load().moe_layer_forward(
        ctypes.byref(desc), _ptr(x), _ptr(w_router), _ptr(bias), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
        _ptr(token_class), int(seed) & 0xFFFFFFFF, _ptr(buf.logits), _ptr(buf.scores), _ptr(buf.topk_idx),
        _ptr(buf.topk_score), _ptr(buf.expert_count), _ptr(buf.seg_count), _ptr(buf.expert_offset),
        _ptr(buf.row_token), _ptr(buf.row_weight), _ptr(buf.pair_row), _ptr(buf.yp), _ptr(buf.y), _ptr(ws),
        ws.numel() * ws.element_size(), _stream(stream)), "moe_layer_forward")
    return buf.y


def moe_profile_attach(table: "MoeProfile | None"):
    """Attach the caller's profile table to this thread (None detaches).  The caller keeps the table alive."""
    _check(load().moe_profile_attach(ctypes.byref(table) if table is not None else None), "moe_profile_attach")


def moe_ffn_schedule_query(desc: MoeDesc, expert_count, compute_units: int = 256):
    """What the tile schedule of the expert GEMMs decides for these rows per expert (host only, nothing is launched):
    ((big tiles, short tiles), [gate/up header of 8 ints, down header of 8 ints])."""
    counts = (ctypes.c_int32 * desc.n_experts)(*[int(c) for c in expert_count])
    tiles = (ctypes.c_int32 * 2)()
    header = (ctypes.c_int32 * 16)()
    _check(load().moe_ffn_schedule_query(ctypes.byref(desc), counts, int(compute_units), tiles, header),
           "moe_ffn_schedule_query")
    return (tiles[0], tiles[1]), [list(header[:8]), list(header[8:])]


def moe_probe_mfma_bf16(blocks: int, iterations: int, sink, random_operands: bool = False, stream=None) -> int:
    """Launch the matrix-core probe; returns the flops of the launch (the caller times it)."""
    flops = ctypes.c_int64(0)
    assert sink.numel() >= blocks * 256
    _check(load().moe_probe_mfma_bf16(int(blocks), int(iterations), int(bool(random_operands)), _ptr(sink),
                                      ctypes.byref(flops), _stream(stream)), "moe_probe_mfma_bf16")
    return int(flops.value)


class LayerBuffers:
    """Device buffers of one layer call, sized by moe_query (allocation only, no arithmetic)."""

    def __init__(self, desc: MoeDesc, device="cuda"):
        import torch

        self.desc = desc
        self.cap, self.slots, self.max_rows, self.workspace_bytes = moe_query(desc)
        n, e, k, d = desc.n_tokens, desc.n_experts, desc.top_k + desc.overselect, desc.d_model
        blocks = desc.device_groups if desc.capacity_scope in (SCOPE_LOCAL, SCOPE_LOCAL_DEVICE) else 1
        act = torch.bfloat16 if desc.dtype == DTYPE_BF16 else torch.float32
        rows = max(self.max_rows, 1)
        i32, f32 = torch.int32, torch.float32
        mk = lambda shape, dt: torch.empty(shape, dtype=dt, device=device)
        self.logits, self.scores = mk((n, e), f32), mk((n, e), f32)
        self.topk_idx, self.topk_score = mk((n, k), i32), mk((n, k), f32)
        self.expert_count, self.seg_count = mk((e,), i32), mk((blocks, e), i32)
        self.expert_offset = mk((e + 1,), i32)
        self.row_token, self.row_weight = mk((rows,), i32), mk((rows,), f32)
        self.pair_row = mk((n, self.slots), i32)
        self.xp, self.yp = mk((rows, d), act), mk((rows, d), act)
        self.y = mk((n, d), act)
        self.workspace = mk((max(self.workspace_bytes, 256),), torch.uint8)


def layer_forward(buf: LayerBuffers, x, w_router, bias, w_gate, w_up, w_down, given_logits=None, stream=None,
                  fused_dispatch=False, token_class=None, seed=0):
    """The calls of one layer, enqueued back to back on one stream; returns buf.y.

    fused_dispatch=False: the five calls route_topk, capacity_drop, dispatch, grouped_ffn, combine.
    fused_dispatch=True: dispatch and grouped_ffn are replaced by moe_dispatch_ffn (xp is not written).
    """
    d = buf.desc
    if given_logits is not None:
        buf.logits.copy_(given_logits)
    moe_route_topk(d, x, w_router, bias, given_logits is not None, buf.logits, buf.scores, buf.topk_idx,
                   buf.topk_score, buf.workspace, stream)
    if token_class is None and seed == 0:
        moe_capacity_drop(d, buf.scores, buf.topk_idx, buf.expert_count, buf.seg_count, buf.expert_offset,
                          buf.row_token, buf.row_weight, buf.pair_row, buf.workspace, stream)
    else:
        moe_capacity_drop_ranked(d, buf.scores, buf.topk_idx, token_class, seed, buf.expert_count, buf.seg_count,
                                 buf.expert_offset, buf.row_token, buf.row_weight, buf.pair_row, buf.workspace, stream)
    if fused_dispatch:
        moe_dispatch_ffn(d, x, buf.expert_offset, buf.row_token, w_gate, w_up, w_down, buf.yp, buf.workspace, stream)
    else:
        moe_dispatch(d, x, buf.expert_offset, buf.row_token, buf.xp, stream)
        moe_grouped_ffn(d, buf.xp, buf.expert_offset, w_gate, w_up, w_down, buf.yp, buf.workspace, stream)
    moe_combine(d, buf.yp, buf.row_weight, buf.pair_row, buf.y, stream)
    return buf.y


def is_unbounded(gamma) -> bool:
    return math.isinf(gamma)
