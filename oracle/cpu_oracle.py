"""ctypes front end of the CPU oracle (oracle/bigmac_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module.
It takes and returns numpy arrays; inputs are fp32 values already rounded to the run's storage
type, results are fp64 (routing indices int32, logits fp32).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bigmac_oracle.c")
_LIB = os.path.join(_HERE, "libbigmac_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  No fast-math, no contraction: the router order is literal."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-mavx2", "-mfma", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_moe_flops_per_token.restype = ctypes.c_double
        _lib.oracle_a2a_bytes_per_token.restype = ctypes.c_double
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def router_logits(x, w_gate, bias=None):
    x, w_gate, bias = _f32(x), _f32(w_gate), _f32(bias)
    T, d = x.shape
    N = w_gate.shape[1]
    assert w_gate.shape[0] == d and d % 64 == 0
    out = np.empty((T, N), np.float32)
    lib().oracle_router_logits(T, d, N, _p(x), _p(w_gate), _p(bias), _p(out))
    return out


def topk_gate(logits, k):
    logits = _f32(logits)
    T, N = logits.shape
    idx = np.empty((T, k), np.int32)
    gate = np.empty((T, k), np.float64)
    lib().oracle_topk_gate(T, N, k, _p(logits), _p(idx), _p(gate))
    return idx, gate


def route(x, w_gate, bias, k):
    logits = router_logits(x, w_gate, bias)
    idx, gate = topk_gate(logits, k)
    return idx, gate, logits


def permutation(idx, N, capacity=0, want_keep=False):
    """offsets, slot_of, src_of (entries past offsets[N] are -1) and, on request, the keep mask."""
    idx = _i32(idx)
    T, k = idx.shape
    offsets = np.empty(N + 1, np.int32)
    slot_of = np.empty((T, k), np.int32)
    src_of = np.full(T * k, -1, np.int32)
    keep = np.empty((T, k), np.int32)
    lib().oracle_permutation(T, k, N, int(capacity), _p(idx), _p(offsets), _p(slot_of), _p(src_of), _p(keep))
    return (offsets, slot_of, src_of, keep) if want_keep else (offsets, slot_of, src_of)


def dispatch(x_low, slot_of):
    x_low, slot_of = _f32(x_low), _i32(slot_of)
    T, width = x_low.shape
    k = slot_of.shape[1]
    out = np.zeros((T * k, width), np.float32)      # rows no pair maps to (capacity drops) stay zero
    lib().oracle_dispatch(T, k, width, _p(x_low), _p(slot_of), _p(out))
    return out


ROUTE_FULL, ROUTE_LOW_F32, ROUTE_LOW_BF16 = 0, 1, 2   # what the router reads: x, or x' as stored in fp32 / bf16


def expert_rows(x_perm, offsets, w1, w2, want_a=False, b1=None, b2=None):
    x_perm, offsets, w1, w2, b1, b2 = _f32(x_perm), _i32(offsets), _f32(w1), _f32(w2), _f32(b1), _f32(b2)
    N, win, hid = w1.shape
    assert w2.shape == (N, hid, win) and x_perm.shape[1] == win
    rows = x_perm.shape[0]
    a = np.empty((rows, hid), np.float64) if want_a else None
    o = np.empty((rows, win), np.float64)
    assert (b1 is None or b1.shape == (N, hid)) and (b2 is None or b2.shape == (N, win))
    lib().oracle_expert_rows_ext(N, win, hid, _p(offsets), _p(x_perm), _p(w1), _p(w2), _p(b1), _p(b2), _p(a), _p(o))
    return (o, a) if want_a else o


def combine(o_perm, slot_of, gate=None):
    o_perm, slot_of, gate = _f64(o_perm), _i32(slot_of), _f64(gate)
    T, k = slot_of.shape
    width = o_perm.shape[1]
    y = np.empty((T, width), np.float64)
    lib().oracle_combine(T, k, width, _p(o_perm), _p(slot_of), _p(gate), _p(y))
    return y


def bigmac_forward(x, w_gate, bias, w_down, w_up, w1, w2, k, sel=None, want_y_low=False, keep=None,
                   b1=None, b2=None, route_low=ROUTE_FULL):
    """route_low != ROUTE_FULL: the router reads the stored x' and w_gate is [r, N]; b1 [N, h], b2 [N, r]:
    expert biases."""
    x, w_gate, bias, w_down, w_up, w1, w2, b1, b2 = map(_f32, (x, w_gate, bias, w_down, w_up, w1, w2, b1, b2))
    T, d = x.shape
    r = w_down.shape[1]
    N, _, h = w1.shape
    assert w_down.shape == (d, r) and w_up.shape == (r, d) and w1.shape == (N, r, h) and w2.shape == (N, h, r)
    assert w_gate.shape == ((r, N) if route_low else (d, N))
    assert (b1 is None or b1.shape == (N, h)) and (b2 is None or b2.shape == (N, r))
    sel = _i32(sel)
    nsel = T if sel is None else sel.shape[0]
    y = np.empty((nsel, d), np.float64)
    y_low = np.empty((nsel, r), np.float64) if want_y_low else None
    lib().oracle_bigmac_forward_ext(T, d, r, N, k, h, _p(x), _p(w_gate), _p(bias), _p(w_down), _p(w_up),
                                    _p(w1), _p(w2), _p(b1), _p(b2), int(route_low), nsel, _p(sel), _p(_i32(keep)),
                                    _p(y), _p(y_low))
    return (y, y_low) if want_y_low else y


def stored_low(x, w_down, mode=ROUTE_LOW_BF16):
    """x' = x W_down as it is stored (fp32, or bf16 for ROUTE_LOW_BF16): what the router of the
    x'-variant reads."""
    x, w_down = _f32(x), _f32(w_down)
    T, d = x.shape
    r = w_down.shape[1]
    out = np.empty((T, r), np.float32)
    lib().oracle_stored_low(T, d, r, _p(x), _p(w_down), int(mode), _p(out))
    return out


def route_low(x, w_down, w_gate, bias, k, mode=ROUTE_LOW_BF16):
    """Routing of the variant whose router reads x' (w_gate is [r, N]): idx, gate, logits, x'."""
    xl = stored_low(x, w_down, mode)
    return route(xl, w_gate, bias, k) + (xl,)


def cdac_forward(x, w_gate, bias, wdn, wup, k, sel=None, keep=None):
    x, w_gate, bias, wdn, wup = map(_f32, (x, w_gate, bias, wdn, wup))
    T, d = x.shape
    N, _, r = wdn.shape
    assert wdn.shape == (N, d, r) and wup.shape == (N, r, d)
    sel = _i32(sel)
    nsel = T if sel is None else sel.shape[0]
    y = np.empty((nsel, d), np.float64)
    lib().oracle_cdac_forward(T, d, r, N, k, _p(x), _p(w_gate), _p(bias), _p(wdn), _p(wup),
                              nsel, _p(sel), _p(_i32(keep)), _p(y))
    return y


def bigmac_backward(x, dy, w_gate, bias, w_down, w_up, w1, w2, k, sel=None, init=None, keep=None,
                    b1=None, b2=None, route_low=ROUTE_FULL):
    """Returns dict(dx, d_w_down, d_w_up, d_w_gate, d_w1, d_w2[, d_b1, d_b2]).  init: optional dict of
    starting values the weight gradients are added to (default zeros)."""
    x, dy, w_gate, bias, w_down, w_up, w1, w2, b1, b2 = map(_f32, (x, dy, w_gate, bias, w_down, w_up, w1, w2, b1, b2))
    T, d = x.shape
    r = w_down.shape[1]
    N, _, h = w1.shape
    sel = _i32(sel)
    nsel = T if sel is None else sel.shape[0]
    init = init or {}
    g = {
        "dx": np.zeros((T, d), np.float64),
        "d_w_down": _f64(init.get("d_w_down", np.zeros((d, r)))).copy(),
        "d_w_up": _f64(init.get("d_w_up", np.zeros((r, d)))).copy(),
        "d_w_gate": _f64(init.get("d_w_gate", np.zeros((r if route_low else d, N)))).copy(),
        "d_w1": _f64(init.get("d_w1", np.zeros((N, r, h)))).copy(),
        "d_w2": _f64(init.get("d_w2", np.zeros((N, h, r)))).copy(),
    }
    if b1 is not None:
        g["d_b1"] = _f64(init.get("d_b1", np.zeros((N, h)))).copy()
    if b2 is not None:
        g["d_b2"] = _f64(init.get("d_b2", np.zeros((N, r)))).copy()
    lib().oracle_bigmac_backward_ext(T, d, r, N, k, h, _p(x), _p(dy), _p(w_gate), _p(bias), _p(w_down),
                                     _p(w_up), _p(w1), _p(w2), _p(b1), _p(b2), int(route_low), nsel, _p(sel),
                                     _p(_i32(keep)), _p(g["dx"]), _p(g["d_w_down"]), _p(g["d_w_up"]), _p(g["d_w_gate"]),
                                     _p(g["d_w1"]), _p(g["d_w2"]), _p(g.get("d_b1")), _p(g.get("d_b2")))
    return g


def cdac_backward(x, dy, w_gate, bias, wdn, wup, k, sel=None, keep=None):
    x, dy, w_gate, bias, wdn, wup = map(_f32, (x, dy, w_gate, bias, wdn, wup))
    T, d = x.shape
    N, _, r = wdn.shape
    sel = _i32(sel)
    nsel = T if sel is None else sel.shape[0]
    g = {"dx": np.zeros((T, d), np.float64), "d_w_gate": np.zeros((d, N), np.float64),
         "d_w1": np.zeros((N, d, r), np.float64), "d_w2": np.zeros((N, r, d), np.float64)}
    lib().oracle_cdac_backward(T, d, r, N, k, _p(x), _p(dy), _p(w_gate), _p(bias), _p(wdn), _p(wup),
                               nsel, _p(sel), _p(_i32(keep)), _p(g["dx"]), _p(g["d_w_gate"]), _p(g["d_w1"]), _p(g["d_w2"]))
    return g


def aux_loss(logits, idx, alpha):
    """Load-balance loss.  The paper names the type and the coefficient (Table 5: aux_loss, 0.001)
    but prints no formula; this is the usual one, written out:  alpha * N * sum_e f_e * P_e  with
    f_e the share of the T*k routed pairs that chose expert e (before any capacity drop) and P_e
    the mean over tokens of softmax(logits[t])[e] over all N experts.  Plain numpy, fp64.
    Returns loss, f [N] and dlogits [T, N], the gradient with f held fixed."""
    z = np.asarray(logits, np.float64)
    idx = np.asarray(idx)
    T, N = z.shape
    p = np.exp(z - z.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    f = np.bincount(idx.ravel(), minlength=N).astype(np.float64) / idx.size
    P = p.sum(axis=0) / T
    loss = float(alpha * N * np.dot(f, P))
    dlogits = alpha * N / T * p * (f[None, :] - (p @ f)[:, None])
    return loss, f, dlogits


def aux_loss_layer_terms(x, w_gate, dlogits):
    """What the loss adds to the layer's gradients: d_w_gate += x^T dlogits, dx += dlogits w_gate^T."""
    x, w_gate = np.asarray(x, np.float64), np.asarray(w_gate, np.float64)
    return {"d_w_gate": x.T @ dlogits, "dx": dlogits @ w_gate.T}


def moe_flops_per_token(d, r, k, bigmac):
    return lib().oracle_moe_flops_per_token(int(d), int(r), int(k), int(bool(bigmac)))


def a2a_bytes_per_token(d, r, k, bigmac, e_b=2):
    return lib().oracle_a2a_bytes_per_token(int(d), int(r), int(k), int(bool(bigmac)), int(e_b))
