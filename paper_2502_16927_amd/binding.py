"""Thin ctypes binding of libbigmac.so: same entry points as include/bigmac.h, torch tensors in.

Argument marshalling only - every step of the layer runs in the library's HIP kernels.  torch is
used for device memory and the current stream.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

F32, BF16 = 0, 1
ORDER_DCCA, ORDER_CDAC = 0, 1
FLAG_ACCUMULATE, FLAG_OUT_BF16, FLAG_WIRE_BF16, FLAG_TILES_LARGE, FLAG_TILES_SMALL, FLAG_ROUTE_LOW, FLAG_NO_FUSED_DISPATCH = 1, 2, 4, 8, 16, 32, 64
WS_ROUTE, WS_DISPATCH, WS_GROUPED_FFN, WS_LAYER_FORWARD, WS_LAYER_TRAIN, WS_SAVED, WS_AUX_LOSS = range(7)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libbigmac.so")
_lib = None


class Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("T", "d", "r", "N", "k", "h", "dtype", "act", "order", "flags", "capacity")] + [
        ("aux_alpha", ctypes.c_float)]


class Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("w_down", "w_up", "w_gate", "gate_bias", "w1", "w2", "b1", "b2")]


class BigmacError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it first (python -m paper_2502_16927_amd.build)")
        L = ctypes.CDLL(_LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        dp = ctypes.POINTER(Dims)
        L.bigmac_workspace_bytes.restype = sz
        L.bigmac_workspace_bytes.argtypes = [dp, ci]
        L.bigmac_status_string.restype = ctypes.c_char_p
        L.bigmac_status_string.argtypes = [ci]
        L.bigmac_forward_matrix_flops.restype = ctypes.c_double
        L.bigmac_forward_matrix_flops.argtypes = [dp]
        L.bigmac_permute_bytes.restype = ctypes.c_double
        L.bigmac_permute_bytes.argtypes = [dp]
        L.bigmac_saved_layout.restype = ci
        L.bigmac_saved_layout.argtypes = [dp] + [ctypes.POINTER(sz)] * 4
        L.bigmac_saved_aux_layout.restype = ci
        L.bigmac_saved_aux_layout.argtypes = [dp] + [ctypes.POINTER(sz)] * 2
        L.bigmac_aux_loss.restype = ci
        L.bigmac_aux_loss.argtypes = [dp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.bigmac_route.restype = ci
        L.bigmac_route.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.bigmac_dispatch.restype = ci
        L.bigmac_dispatch.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.bigmac_dispatch_static.restype = ci
        L.bigmac_dispatch_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        L.bigmac_grouped_ffn.restype = ci
        L.bigmac_grouped_ffn.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.bigmac_combine.restype = ci
        L.bigmac_combine.argtypes = [dp, vp, vp, vp, vp, vp]
        L.bigmac_layer_forward.restype = ci
        L.bigmac_layer_forward.argtypes = [dp, ctypes.POINTER(Params), vp, vp, vp, vp, sz, vp]
        L.bigmac_layer_backward.restype = ci
        L.bigmac_layer_backward.argtypes = [dp, ctypes.POINTER(Params), vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.bigmac_set_stage_events.restype = ci
        L.bigmac_set_stage_events.argtypes = [ctypes.POINTER(vp)]
        L.bigmac_dispatch_folding.restype = ci
        L.bigmac_dispatch_folding.argtypes = [dp, ci]
        L.bigmac_stage_name.restype = ctypes.c_char_p
        L.bigmac_stage_name.argtypes = [ci]
        L.bigmac_gather_probe.restype = ci
        L.bigmac_gather_probe.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int64, ci, vp, vp]
        L.bigmac_mfma_probe.restype = ci
        L.bigmac_mfma_probe.argtypes = [ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
        _lib = L
    return _lib


EXPORTS = ("bigmac_workspace_bytes", "bigmac_status_string", "bigmac_forward_matrix_flops", "bigmac_permute_bytes",
           "bigmac_saved_layout", "bigmac_saved_aux_layout", "bigmac_aux_loss", "bigmac_route", "bigmac_dispatch", "bigmac_dispatch_static", "bigmac_grouped_ffn", "bigmac_combine",
           "bigmac_layer_forward", "bigmac_layer_backward", "bigmac_set_stage_events", "bigmac_stage_name", "bigmac_dispatch_folding",
           "bigmac_mfma_probe", "bigmac_gather_probe")
STAGE_COUNT = 22


def make_dims(T, d, r, N, k, h, dtype=BF16, order=ORDER_DCCA, flags=0, act=0, capacity=0, aux_alpha=0.0) -> Dims:
    return Dims(T, d, r, N, k, h, dtype, act, order, flags, capacity, aux_alpha)


def dims_of(wl, order=ORDER_DCCA, flags=0, capacity=0, aux_alpha=0.0) -> Dims:
    return make_dims(wl.T, wl.d, wl.r, wl.N, wl.k, wl.h, wl.dtype, order, flags, capacity=capacity, aux_alpha=aux_alpha)


def expert_capacity(T: int, k: int, N: int, factor: float) -> int:
    """Rows an expert keeps at capacity factor `factor`: ceil(factor * T * k / N)."""
    return -(-int(round(factor * 1e6)) * T * k // (N * 1000000))


def status_string(status: int) -> str:
    return lib().bigmac_status_string(status).decode()


def workspace_bytes(dims: Dims, kind: int) -> int:
    return lib().bigmac_workspace_bytes(ctypes.byref(dims), kind)


def forward_matrix_flops(dims: Dims) -> float:
    return lib().bigmac_forward_matrix_flops(ctypes.byref(dims))


def permute_bytes(dims: Dims) -> float:
    return lib().bigmac_permute_bytes(ctypes.byref(dims))


def saved_layout(dims: Dims) -> dict:
    offs = [ctypes.c_size_t() for _ in range(4)]
    _check(lib().bigmac_saved_layout(ctypes.byref(dims), *[ctypes.byref(o) for o in offs]), "bigmac_saved_layout")
    return dict(zip(("topk_idx", "topk_w", "expert_offsets", "slot_of"), (o.value for o in offs)))


def saved_aux_layout(dims: Dims) -> dict:
    offs = [ctypes.c_size_t() for _ in range(2)]
    _check(lib().bigmac_saved_aux_layout(ctypes.byref(dims), *[ctypes.byref(o) for o in offs]), "bigmac_saved_aux_layout")
    return dict(zip(("aux_loss", "aux_share"), (o.value for o in offs)))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous(), "the library takes contiguous tensors"
    return t.data_ptr()


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return stream


def _check(rc: int, where: str):
    if rc != 0:
        raise BigmacError(rc, where)


def make_params(w_down, w_up, w_gate, gate_bias, w1, w2, b1=None, b2=None) -> Params:
    return Params(_ptr(w_down), _ptr(w_up), _ptr(w_gate), _ptr(gate_bias), _ptr(w1), _ptr(w2), _ptr(b1), _ptr(b2))


def bigmac_aux_loss(dims, logits, topk_idx, loss, share, dlogits=None, ws=None, stream=None):
    _check(lib().bigmac_aux_loss(ctypes.byref(dims), _ptr(logits), _ptr(topk_idx), _ptr(loss), _ptr(share), _ptr(dlogits),
                                 _ptr(ws), _nbytes(ws), _stream(stream)), "bigmac_aux_loss")


def bigmac_route(dims, x, w_gate, gate_bias, topk_idx, topk_w, logits_out=None, ws=None, stream=None):
    _check(lib().bigmac_route(ctypes.byref(dims), _ptr(x), _ptr(w_gate), _ptr(gate_bias), _ptr(topk_idx), _ptr(topk_w),
                              _ptr(logits_out), _ptr(ws), _nbytes(ws), _stream(stream)), "bigmac_route")


def bigmac_dispatch(dims, x_low, topk_idx, x_perm, expert_offsets, slot_of, src_of, ws, stream=None):
    _check(lib().bigmac_dispatch(ctypes.byref(dims), _ptr(x_low), _ptr(topk_idx), _ptr(x_perm), _ptr(expert_offsets),
                                 _ptr(slot_of), _ptr(src_of), _ptr(ws), _nbytes(ws), _stream(stream)), "bigmac_dispatch")


def bigmac_dispatch_static(dims, x_low, topk_idx, x_perm, expert_offsets, slot_of, src_of, stream=None):
    _check(lib().bigmac_dispatch_static(ctypes.byref(dims), _ptr(x_low), _ptr(topk_idx), _ptr(x_perm), _ptr(expert_offsets),
                                        _ptr(slot_of), _ptr(src_of), _stream(stream)), "bigmac_dispatch_static")


def bigmac_grouped_ffn(dims, x_perm, expert_offsets, w1, w2, act_saved, o_perm, ws, stream=None, b1=None, b2=None):
    _check(lib().bigmac_grouped_ffn(ctypes.byref(dims), _ptr(x_perm), _ptr(expert_offsets), _ptr(w1), _ptr(w2), _ptr(b1), _ptr(b2),
                                    _ptr(act_saved), _ptr(o_perm), _ptr(ws), _nbytes(ws), _stream(stream)), "bigmac_grouped_ffn")


def bigmac_combine(dims, o_perm, slot_of, topk_w, y_low, stream=None):
    _check(lib().bigmac_combine(ctypes.byref(dims), _ptr(o_perm), _ptr(slot_of), _ptr(topk_w), _ptr(y_low),
                                _stream(stream)), "bigmac_combine")


def bigmac_gather_probe(table, order, rows, row_bytes, streaming, sink, stream=None) -> None:
    _check(lib().bigmac_gather_probe(_ptr(table), _ptr(order), int(rows), int(row_bytes), int(bool(streaming)), _ptr(sink), _stream(stream)),
           "bigmac_gather_probe")


def bigmac_mfma_probe(blocks, iters, sink, stream=None) -> float:
    """Enqueues the matrix-core rate probe; returns the flops of the launch (the caller times it)."""
    flops = ctypes.c_double(0.0)
    _check(lib().bigmac_mfma_probe(int(blocks), int(iters), _ptr(sink), ctypes.byref(flops), _stream(stream)), "bigmac_mfma_probe")
    return flops.value


def bigmac_layer_forward(dims, params, x, y, saved, ws, stream=None):
    _check(lib().bigmac_layer_forward(ctypes.byref(dims), ctypes.byref(params), _ptr(x), _ptr(y), _ptr(saved), _ptr(ws),
                                      _nbytes(ws), _stream(stream)), "bigmac_layer_forward")


def bigmac_layer_backward(dims, params, x, dy, saved, dx, d_w_down, d_w_up, d_w_gate, d_w1, d_w2, ws, stream=None,
                          d_b1=None, d_b2=None):
    _check(lib().bigmac_layer_backward(ctypes.byref(dims), ctypes.byref(params), _ptr(x), _ptr(dy), _ptr(saved), _ptr(dx),
                                       _ptr(d_w_down), _ptr(d_w_up), _ptr(d_w_gate), _ptr(d_w1), _ptr(d_w2), _ptr(d_b1), _ptr(d_b2),
                                       _ptr(ws), _nbytes(ws), _stream(stream)), "bigmac_layer_backward")


def dispatch_folding(dims, training: bool) -> int:
    """0: copy kernel; 1: folded into the expert-up product; 2: folded into the descending projection."""
    rc = lib().bigmac_dispatch_folding(ctypes.byref(dims), int(bool(training)))
    if rc < 0:
        _check(rc, "bigmac_dispatch_folding")
    return rc


def stage_name(stage: int) -> str:
    return lib().bigmac_stage_name(stage).decode()


class StageEvents:
    """A table of 2 * STAGE_COUNT timing events (torch events, so they live on torch's runtime)
    that the layer calls record around each stage while the table is installed."""

    def __init__(self):
        self.events = [torch.cuda.Event(enable_timing=True) for _ in range(2 * STAGE_COUNT)]
        for e in self.events:
            e.record()                       # materialise the underlying hipEvent_t
        self.table = (ctypes.c_void_p * (2 * STAGE_COUNT))(*[e.cuda_event for e in self.events])

    def install(self):
        _check(lib().bigmac_set_stage_events(self.table), "bigmac_set_stage_events")

    @staticmethod
    def clear():
        _check(lib().bigmac_set_stage_events(None), "bigmac_set_stage_events")

    def elapsed_ms(self, recorded: set) -> dict:
        """Per-stage milliseconds for the stages in `recorded` (call after a synchronize)."""
        return {s: self.events[2 * s].elapsed_time(self.events[2 * s + 1]) for s in recorded}


# ----------------------------------------------------------------- device buffers (allocation only)

def to_device(a, dtype_code, device="cuda:0"):
    """numpy fp32 array (already rounded to the storage type) -> device tensor of that type."""
    if a is None:
        return None
    t = torch.from_numpy(a).to(device)
    return t.to(torch.bfloat16) if dtype_code == BF16 else t


def act_dtype(dtype_code):
    return torch.bfloat16 if dtype_code == BF16 else torch.float32


def alloc_bytes(n, device="cuda:0"):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)
