"""ctypes binding of the C ABI in include/moe.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libmoe_gfx950.so. PyTorch is used for device memory and streams, nothing else. There is no
CPU fallback: if the library is missing and cannot be built, importing callers get an error.

The functions mirror the C entry points (moe_create, moe_pack_weights, moe_route,
moe_dispatch, moe_expert_ffn, moe_combine); `MoEPath` strings the four hot calls together
over buffers it allocates once.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # imported before the library so both share one HIP runtime (same SONAME)

from . import build as _build

MOE_OK, MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_HIP = 0, 1, 2, 3
MOE_F32, MOE_BF16 = 0, 1
_DTYPES = {"f32": (MOE_F32, torch.float32), "bf16": (MOE_BF16, torch.bfloat16)}

EXPORTS = ("moe_create", "moe_destroy", "moe_last_error", "moe_status_string", "moe_ffn_kernel_name", "moe_packed_weight_bytes",
           "moe_pack_weights", "moe_route", "moe_gate_route", "moe_dispatch", "moe_expert_ffn", "moe_ffn_input", "moe_ffn_output",
           "moe_combine", "moe_plan_experts", "moe_slot_segments", "moe_expert_ffn_segments", "moe_route_dispatch",
           "moe_gate_route_dispatch", "moe_expert_ffn_static", "moe_probe_stream_read", "moe_probe_mfma")


class MoeConfig(ctypes.Structure):
    _fields_ = [("T_max", ctypes.c_int32), ("d", ctypes.c_int32), ("f", ctypes.c_int32),
                ("E", ctypes.c_int32), ("k", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("load_skew", ctypes.c_float)]


class MoeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"moe status {status}: {message}")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libmoe_gfx950.so. It is built first if no built library exists or if the one that
    exists was built from other sources than the tree holds now (build.py keeps a hash of the
    sources beside the library), so an edited kernel never runs from a stale binary."""
    global _lib
    if _lib is not None:
        return _lib
    if not _build.is_current():
        _build.build()
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, i32, cfgp = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(MoeConfig)
    lib.moe_create.argtypes = [cfgp, ctypes.POINTER(vp)]
    lib.moe_create.restype = ctypes.c_int
    lib.moe_destroy.argtypes = [vp]
    lib.moe_destroy.restype = None
    lib.moe_last_error.argtypes = [vp]
    lib.moe_last_error.restype = ctypes.c_char_p
    lib.moe_status_string.argtypes = [ctypes.c_int]
    lib.moe_status_string.restype = ctypes.c_char_p
    lib.moe_ffn_kernel_name.argtypes = [vp, i32, i32]
    lib.moe_ffn_kernel_name.restype = ctypes.c_char_p
    lib.moe_packed_weight_bytes.argtypes = [cfgp]
    lib.moe_packed_weight_bytes.restype = ctypes.c_size_t
    lib.moe_pack_weights.argtypes = [vp] + [vp] * 4 + [vp]
    lib.moe_route.argtypes = [vp, i32] + [vp] * 5 + [vp]
    lib.moe_gate_route.argtypes = [vp, i32] + [vp] * 7 + [vp]
    lib.moe_dispatch.argtypes = [vp, i32] + [vp] * 6 + [vp]
    lib.moe_route_dispatch.argtypes = [vp, i32] + [vp] * 9 + [vp]
    lib.moe_gate_route_dispatch.argtypes = [vp, i32] + [vp] * 10 + [vp]
    lib.moe_gate_route_dispatch.restype = ctypes.c_int
    lib.moe_expert_ffn.argtypes = [vp, i32] + [vp] * 5 + [vp]
    lib.moe_expert_ffn_static.argtypes = [vp, i32] + [vp] * 4 + [vp]
    lib.moe_expert_ffn_static.restype = ctypes.c_int
    lib.moe_ffn_input.argtypes = [vp, i32] + [vp] * 4 + [vp]
    lib.moe_ffn_output.argtypes = [vp, i32] + [vp] * 4 + [vp]
    lib.moe_combine.argtypes = [vp, i32] + [vp] * 4 + [vp]
    dp, ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)
    lib.moe_plan_experts.argtypes = [i32, i32, i32, dp, ctypes.c_double, ip, ip, ip, dp]
    lib.moe_slot_segments.argtypes = [vp, i32] + [vp] * 6 + [vp]
    lib.moe_expert_ffn_segments.argtypes = [vp, i32, i32, i32] + [vp] * 7 + [vp]
    lib.moe_probe_stream_read.argtypes = [vp, vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_size_t), vp]
    lib.moe_probe_mfma.argtypes = [vp, vp, i32, i32, vp, dp, vp]
    lib.moe_probe_stream_read.restype = lib.moe_probe_mfma.restype = ctypes.c_int
    for name in ("moe_pack_weights", "moe_route", "moe_gate_route", "moe_dispatch", "moe_expert_ffn", "moe_ffn_input", "moe_ffn_output",
           "moe_combine", "moe_plan_experts", "moe_slot_segments", "moe_expert_ffn_segments", "moe_route_dispatch"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def library_source_hash() -> str:
    """Hash of the sources the loaded library was built from (as build.py recorded it)."""
    load_library()
    try:
        with open(_build.STAMP_PATH) as fh:
            return fh.read().strip()
    except OSError:
        return ""


def _ptr(t) -> Optional[int]:
    """Device address of a tensor (or a raw int address, or None)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _check(ctx, status: int):
    if status != MOE_OK:
        lib = load_library()
        msg = lib.moe_last_error(ctx).decode() if ctx else ""
        raise MoeError(status, f"{lib.moe_status_string(status).decode()} {msg}".strip())


def moe_create(T_max: int, d: int, f: int, E: int, k: int, dtype: str, load_skew: float = 0.0) -> int:
    lib = load_library()
    cfg = MoeConfig(T_max, d, f, E, k, _DTYPES[dtype][0], load_skew)
    ctx = ctypes.c_void_p()
    status = lib.moe_create(ctypes.byref(cfg), ctypes.byref(ctx))
    if status != MOE_OK:
        raise MoeError(status, lib.moe_status_string(status).decode())
    return ctx.value


def moe_destroy(ctx: int) -> None:
    load_library().moe_destroy(ctx)


def moe_ffn_kernel_name(ctx, T: int, stage: int) -> str:
    return load_library().moe_ffn_kernel_name(ctx, T, stage).decode()


def moe_packed_weight_bytes(T_max: int, d: int, f: int, E: int, k: int, dtype: str) -> int:
    cfg = MoeConfig(T_max, d, f, E, k, _DTYPES[dtype][0])
    return load_library().moe_packed_weight_bytes(ctypes.byref(cfg))


def moe_pack_weights(ctx, w_gate, w_up, w_down, packed, stream=None) -> None:
    _check(ctx, load_library().moe_pack_weights(ctx, _ptr(w_gate), _ptr(w_up), _ptr(w_down), _ptr(packed),
                                                _stream(stream)))


def moe_route(ctx, T, logits, topk_idx, topk_w, counts, offsets, stream=None) -> None:
    _check(ctx, load_library().moe_route(ctx, T, _ptr(logits), _ptr(topk_idx), _ptr(topk_w), _ptr(counts),
                                         _ptr(offsets), _stream(stream)))


def moe_gate_route(ctx, T, x, w_router, logits, topk_idx, topk_w, counts, offsets, stream=None) -> None:
    _check(ctx, load_library().moe_gate_route(ctx, T, _ptr(x), _ptr(w_router), _ptr(logits), _ptr(topk_idx),
                                              _ptr(topk_w), _ptr(counts), _ptr(offsets), _stream(stream)))


def moe_dispatch(ctx, T, x, topk_idx, offsets, xp, pos, src, stream=None) -> None:
    _check(ctx, load_library().moe_dispatch(ctx, T, _ptr(x), _ptr(topk_idx), _ptr(offsets), _ptr(xp), _ptr(pos),
                                            _ptr(src), _stream(stream)))


def moe_route_dispatch(ctx, T, logits, x, topk_idx, topk_w, counts, offsets, xp, pos, src, stream=None) -> None:
    _check(ctx, load_library().moe_route_dispatch(ctx, T, _ptr(logits), _ptr(x), _ptr(topk_idx), _ptr(topk_w),
                                                  _ptr(counts), _ptr(offsets), _ptr(xp), _ptr(pos), _ptr(src),
                                                  _stream(stream)))


def moe_gate_route_dispatch(ctx, T, x, w_router, logits, topk_idx, topk_w, counts, offsets, xp, pos, src,
                            stream=None) -> None:
    _check(ctx, load_library().moe_gate_route_dispatch(ctx, T, _ptr(x), _ptr(w_router), _ptr(logits), _ptr(topk_idx),
                                                       _ptr(topk_w), _ptr(counts), _ptr(offsets), _ptr(xp), _ptr(pos),
                                                       _ptr(src), _stream(stream)))


def moe_expert_ffn(ctx, T, xp, offsets, packed_w, h_ws, y, stream=None) -> None:
    _check(ctx, load_library().moe_expert_ffn(ctx, T, _ptr(xp), _ptr(offsets), _ptr(packed_w), _ptr(h_ws), _ptr(y),
                                              _stream(stream)))


def moe_expert_ffn_static(ctx, T, xp, offsets, packed_w, y, stream=None) -> None:
    _check(ctx, load_library().moe_expert_ffn_static(ctx, T, _ptr(xp), _ptr(offsets), _ptr(packed_w), _ptr(y),
                                                     _stream(stream)))


def moe_ffn_input(ctx, T, xp, offsets, packed_w, h, stream=None) -> None:
    _check(ctx, load_library().moe_ffn_input(ctx, T, _ptr(xp), _ptr(offsets), _ptr(packed_w), _ptr(h), _stream(stream)))


def moe_ffn_output(ctx, T, h, offsets, packed_w, y, stream=None) -> None:
    _check(ctx, load_library().moe_ffn_output(ctx, T, _ptr(h), _ptr(offsets), _ptr(packed_w), _ptr(y), _stream(stream)))


def moe_combine(ctx, T, y, pos, topk_w, out, stream=None) -> None:
    _check(ctx, load_library().moe_combine(ctx, T, _ptr(y), _ptr(pos), _ptr(topk_w), _ptr(out), _stream(stream)))


def moe_plan_experts(a, K: float, N: int, S: int):
    """Host call (no GPU): returns (replicas[M], slots, node_cost[N]); slots[j] lists node j's
    (expert, copy) pairs in placement order."""
    M = len(a)
    arr = (ctypes.c_double * M)(*[float(v) for v in a])
    replicas = (ctypes.c_int32 * M)()
    slot_expert = (ctypes.c_int32 * (N * S))()
    slot_copy = (ctypes.c_int32 * (N * S))()
    cost = (ctypes.c_double * N)()
    lib = load_library()
    status = lib.moe_plan_experts(M, N, S, arr, float(K), replicas, slot_expert, slot_copy, cost)
    if status != MOE_OK:
        raise MoeError(status, lib.moe_status_string(status).decode())
    slots = [[(slot_expert[j * S + q], slot_copy[j * S + q]) for q in range(S) if slot_expert[j * S + q] >= 0]
             for j in range(N)]
    return list(replicas), slots, list(cost)


def moe_slot_segments(ctx, n_slots, slot_expert, slot_copy, replicas, offsets, seg_begin, seg_end, stream=None) -> None:
    _check(ctx, load_library().moe_slot_segments(ctx, n_slots, _ptr(slot_expert), _ptr(slot_copy), _ptr(replicas),
                                                 _ptr(offsets), _ptr(seg_begin), _ptr(seg_end), _stream(stream)))


def moe_expert_ffn_segments(ctx, T, n_segs, rows_hint, xp, seg_begin, seg_end, seg_expert, packed_w, h_ws, y,
                            stream=None) -> None:
    _check(ctx, load_library().moe_expert_ffn_segments(ctx, T, n_segs, rows_hint, _ptr(xp), _ptr(seg_begin),
                                                       _ptr(seg_end), _ptr(seg_expert), _ptr(packed_w), _ptr(h_ws),
                                                       _ptr(y), _stream(stream)))


def moe_probe_stream_read(ctx, buf, nbytes, sink, stream=None) -> int:
    """Enqueue the streaming-read probe over buf[:nbytes]; returns the bytes it reads."""
    got = ctypes.c_size_t(0)
    _check(ctx, load_library().moe_probe_stream_read(ctx, _ptr(buf), nbytes, _ptr(sink), ctypes.byref(got),
                                                     _stream(stream)))
    return got.value


def moe_probe_mfma(ctx, operands, iters, workgroups, sink, stream=None) -> float:
    """Enqueue the register-only MFMA probe; returns the flops of the launch."""
    flops = ctypes.c_double(0.0)
    _check(ctx, load_library().moe_probe_mfma(ctx, _ptr(operands), iters, workgroups, _ptr(sink), ctypes.byref(flops),
                                              _stream(stream)))
    return flops.value


class NodeShare:
    """One expert node's slots under an expert plan: device copies of its (expert, copy) list and
    the row ranges moe_slot_segments derives from a batch's offsets."""

    def __init__(self, node_slots, replicas, device):
        i32 = torch.int32
        self.n = len(node_slots)
        n = max(self.n, 1)
        self.slot_expert = torch.tensor([e for e, _ in node_slots] or [0], dtype=i32, device=device)
        self.slot_copy = torch.tensor([r for _, r in node_slots] or [0], dtype=i32, device=device)
        self.replicas = torch.tensor(list(replicas), dtype=i32, device=device)
        self.seg_begin = torch.zeros(n, dtype=i32, device=device)
        self.seg_end = torch.zeros(n, dtype=i32, device=device)


class MoEPath:
    """Buffers for one (T_max, d, f, E, k, dtype) layer plus the four hot calls over them."""

    def __init__(self, T_max: int, d: int, f: int, E: int, k: int, dtype: str, device="cuda:0", load_skew: float = 0.0):
        if not torch.cuda.is_available():
            raise RuntimeError("MoEPath needs a GPU: there is no CPU path")
        self.T_max, self.d, self.f, self.E, self.k, self.dtype = T_max, d, f, E, k, dtype
        self.device = torch.device(device)
        self.tdtype = _DTYPES[dtype][1]
        self.ctx = moe_create(T_max, d, f, E, k, dtype, load_skew)
        A = max(T_max * k, 1)
        dev, i32 = self.device, torch.int32
        self.topk_idx = torch.empty((max(T_max, 1), k), dtype=i32, device=dev)
        self.topk_w = torch.empty((max(T_max, 1), k), dtype=torch.float32, device=dev)
        self.counts = torch.empty(E, dtype=i32, device=dev)
        self.offsets = torch.empty(E + 1, dtype=i32, device=dev)
        self.xp = torch.empty((A, d), dtype=self.tdtype, device=dev)
        self.pos = torch.empty((max(T_max, 1), k), dtype=i32, device=dev)
        self.src = torch.empty(A, dtype=i32, device=dev)
        self.h = torch.empty((A, f), dtype=self.tdtype, device=dev)
        self.y = torch.empty((A, d), dtype=self.tdtype, device=dev)
        self.out = torch.empty((max(T_max, 1), d), dtype=self.tdtype, device=dev)
        self.packed = None

    def close(self):
        if self.ctx:
            moe_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def pack_weights(self, w_gate, w_up, w_down, stream=None):
        """w_gate/w_up [E, f, d], w_down [E, d, f] device tensors in the layer dtype."""
        nbytes = moe_packed_weight_bytes(self.T_max, self.d, self.f, self.E, self.k, self.dtype)
        self.packed = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        moe_pack_weights(self.ctx, w_gate, w_up, w_down, self.packed, stream)
        return self.packed

    def route(self, logits, T=None, stream=None):
        T = logits.shape[0] if T is None else T
        moe_route(self.ctx, T, logits, self.topk_idx, self.topk_w, self.counts, self.offsets, stream)

    def gate_route(self, x, w_router, logits=None, T=None, stream=None):
        T = x.shape[0] if T is None else T
        moe_gate_route(self.ctx, T, x, w_router, logits, self.topk_idx, self.topk_w, self.counts, self.offsets, stream)

    def dispatch(self, x, T=None, stream=None):
        T = x.shape[0] if T is None else T
        moe_dispatch(self.ctx, T, x, self.topk_idx, self.offsets, self.xp, self.pos, self.src, stream)

    def route_dispatch(self, x, logits, T=None, stream=None):
        T = x.shape[0] if T is None else T
        moe_route_dispatch(self.ctx, T, logits, x, self.topk_idx, self.topk_w, self.counts, self.offsets, self.xp,
                           self.pos, self.src, stream)

    def gate_route_dispatch(self, x, w_router, logits=None, T=None, stream=None):
        T = x.shape[0] if T is None else T
        moe_gate_route_dispatch(self.ctx, T, x, w_router, logits, self.topk_idx, self.topk_w, self.counts,
                                self.offsets, self.xp, self.pos, self.src, stream)

    def ffn_kernel_name(self, T, stage) -> str:
        return moe_ffn_kernel_name(self.ctx, T, stage)

    def expert_ffn(self, T, stream=None):
        moe_expert_ffn(self.ctx, T, self.xp, self.offsets, self.packed, self.h, self.y, stream)

    def ffn_input(self, T, stream=None):
        moe_ffn_input(self.ctx, T, self.xp, self.offsets, self.packed, self.h, stream)

    def ffn_output(self, T, stream=None):
        moe_ffn_output(self.ctx, T, self.h, self.offsets, self.packed, self.y, stream)

    def combine(self, T, stream=None):
        moe_combine(self.ctx, T, self.y, self.pos, self.topk_w, self.out, stream)

    def node_share(self, node_slots, replicas) -> NodeShare:
        return NodeShare(node_slots, replicas, self.device)

    def expert_ffn_node(self, T, share: NodeShare, rows_hint=0, stream=None):
        """The expert FFN over one node's slots of an expert plan (after route and dispatch)."""
        moe_slot_segments(self.ctx, share.n, share.slot_expert, share.slot_copy, share.replicas, self.offsets,
                          share.seg_begin, share.seg_end, stream)
        moe_expert_ffn_segments(self.ctx, T, share.n, rows_hint, self.xp, share.seg_begin, share.seg_end,
                                share.slot_expert, self.packed, self.h, self.y, stream)

    def forward_from_gate(self, x, w_router, stream=None):
        """One pass of the path that starts at the gating GEMM: x[T, d], w_router[E, d] float32."""
        T = x.shape[0]
        self.gate_route_dispatch(x, w_router, None, T, stream)
        self.expert_ffn(T, stream)
        self.combine(T, stream)
        return self.out[:T]

    def forward(self, x, logits, stream=None):
        """One pass of the whole hot path; returns out[:T] (a view of the preallocated buffer)."""
        T = x.shape[0]
        self.route_dispatch(x, logits, T, stream)
        self.expert_ffn(T, stream)
        self.combine(T, stream)
        return self.out[:T]
