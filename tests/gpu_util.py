"""Helpers of the GPU parity tests: move seeded inputs to the device, call the C ABI through the
binding, bring results back as numpy.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2502_16927_amd import binding as B
from paper_2502_16927_amd import synth

TOL = 2e-2          # max-abs error relative to the RMS of the oracle tensor (outputs and gradients)
# The layer stores x', act(x' W1) and the expert outputs in bf16 (the dispatched rows and the MFMA
# operands).  Those three roundings alone - emulated on the CPU in fp64 with no GPU code, see
# tests/test_precision_floor.py - put 0.29 % RMS of noise on y whose largest element over a few
# hundred thousand reaches 2.1e-2 of the RMS at the widest shapes (d = 4096, r = 1024), where the
# pre-activations are large enough for the GELU to amplify the rounding of x'.  For those
# workloads the bar on y is 1.25 x TOL; it stays TOL for the others.
TOL_WIDE = 1.25 * TOL


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.abs(np.asarray(gpu, np.float64) - ref).max() / max(rms, 1e-30))


def check_dx(gpu_rows: np.ndarray, ref_rows: np.ndarray, tol: float = TOL):
    """dx on sampled tokens.  dx carries the gate gradient sum_j dlogit_j W_g[:, e_j], whose error is
    a per-token error of dlogit (through the bf16-stored expert outputs) times a per-element
    weight: a product of two Gaussians, with a far heavier tail than the other tensors.  A CPU
    emulation of the pipeline that does nothing but round the stored tensors to bf16 (no GPU code)
    shows the same tail: about 1 token in 300 above 2e-2 of the RMS at the GPT-XL shape.  The bar
    is therefore: every sampled token within 1.5 x tol, and at most 1 % of them above tol."""
    ref_rows = np.asarray(ref_rows, np.float64)
    rms = float(np.sqrt(np.mean(ref_rows * ref_rows)))
    per_token = np.abs(np.asarray(gpu_rows, np.float64) - ref_rows).max(axis=1) / rms
    worst, over = float(per_token.max()), float(np.mean(per_token > tol))
    assert worst < 1.5 * tol and over <= 0.01, f"dx: worst token {worst:.4f}, {over:.2%} of tokens above {tol}"
    return worst, over


def wgrad_err(gpu: np.ndarray, ref: np.ndarray, rows_per_expert: float) -> float:
    """Error measure for a weight gradient.  With many rows per expert every element is a long
    sum and the error is a small Gaussian fraction of the tensor's RMS: the 2e-2 bar applies as
    it stands.  With only a few rows (below 256: degenerate test shapes, token samples) an element is a handful of
    products whose largest values sit far above the RMS, and a bf16 rounding of 2^-9 relative
    on such an element alone exceeds 2e-2 of the RMS; there the error is taken relative to the
    largest element instead."""
    if rows_per_expert >= 256:
        return rel_err(gpu, ref)
    ref = np.asarray(ref, np.float64)
    return float(np.abs(np.asarray(gpu, np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


def check_weight_grads(grads: dict, ref: dict, counts: np.ndarray, T: int, tol: float, dcca: bool = True, scale: float = 1.0):
    """Every parameter matrix against the oracle.  The matrices of one expert (W1[e], W2[e] and
    the expert's gating column W_g[:, e]) are parameters of their own: each is compared with the
    RMS of its own gradient, so that under skewed routing a popular expert's large gradient does
    not set the bar for the others.  An expert without rows must get an exactly zero gradient."""
    worst = {}
    if dcca:
        for n in ("d_w_down", "d_w_up"):
            worst[n] = wgrad_err(grads[n], ref[n], T)
    for n in ("d_w1", "d_w2", "d_w_gate"):
        w = 0.0
        for e, c in enumerate(counts):
            g = grads[n][:, e] if n == "d_w_gate" else grads[n][e]
            r = ref[n][:, e] if n == "d_w_gate" else ref[n][e]
            if c == 0:
                assert not np.any(g) and not np.any(r), f"{n}[{e}]: expert without rows has a gradient"
                continue
            err = wgrad_err(g, r, c)
            if n == "d_w_gate":
                # a gating column fed by a handful of rows is x_t times one scalar dlogit, itself a
                # difference of gate gradients that can cancel: its own size is no yardstick, the
                # whole matrix's RMS (the plain reading of the bar) is
                err = min(err, float(np.abs(g - r).max() / np.sqrt(np.mean(np.asarray(ref[n], np.float64) ** 2))))
            w = max(w, err)
        worst[n] = w
    for n, v in worst.items():
        assert v < tol * scale, f"{n}: {v:.4f} >= {tol * scale}"
    return worst


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


class DeviceLayer:
    """All device buffers of one layer call for a workload (allocation and marshalling only)."""

    def __init__(self, wl: synth.Workload, data: dict, order=B.ORDER_DCCA, flags=0, device="cuda:0", capacity=0, aux_alpha=0.0):
        self.wl, self.order, self.flags, self.device = wl, order, flags, device
        self.dims = B.dims_of(wl, order, flags, capacity=capacity, aux_alpha=aux_alpha)
        dt = wl.dtype
        self.x = B.to_device(data["x"], dt, device)
        self.dy = B.to_device(data.get("dy"), dt, device)
        self.w_gate = B.to_device(data["w_gate"], B.F32, device)
        self.gate_bias = B.to_device(data["gate_bias"], B.F32, device)
        if order == B.ORDER_DCCA:
            self.w_down = B.to_device(data["w_down"], dt, device)
            self.w_up = B.to_device(data["w_up"], dt, device)
            self.w1 = B.to_device(data["w1"], dt, device)
            self.w2 = B.to_device(data["w2"], dt, device)
        else:  # same parameters, swapped roles: first matrix [N, d, r], second [N, r, d]
            self.w_down = self.w_up = None
            self.w1 = B.to_device(data["cdac_w1"], dt, device)
            self.w2 = B.to_device(data["cdac_w2"], dt, device)
        self.params = B.make_params(self.w_down, self.w_up, self.w_gate, self.gate_bias, self.w1, self.w2)
        out_bf16 = dt == B.BF16 and (flags & B.FLAG_OUT_BF16)
        self.out_dtype = torch.bfloat16 if out_bf16 else torch.float32
        self.y = torch.empty((wl.T, wl.d), dtype=self.out_dtype, device=device)
        self.ws_infer = None
        self.ws_train = None
        self.saved = None

    def forward(self, training: bool):
        if training:
            if self.saved is None:
                self.saved = B.alloc_bytes(B.workspace_bytes(self.dims, B.WS_SAVED), self.device)
                self.ws_train = B.alloc_bytes(B.workspace_bytes(self.dims, B.WS_LAYER_TRAIN), self.device)
            B.bigmac_layer_forward(self.dims, self.params, self.x, self.y, self.saved, self.ws_train)
        else:
            if self.ws_infer is None:
                self.ws_infer = B.alloc_bytes(B.workspace_bytes(self.dims, B.WS_LAYER_FORWARD), self.device)
            B.bigmac_layer_forward(self.dims, self.params, self.x, self.y, None, self.ws_infer)
        return self.y

    def alloc_grads(self, init: dict | None = None):
        wl, dev = self.wl, self.device
        win, hid = (wl.r, wl.h) if self.order == B.ORDER_DCCA else (wl.d, wl.r)
        shapes = {"d_w_down": (wl.d, wl.r), "d_w_up": (wl.r, wl.d), "d_w_gate": (wl.d, wl.N),
                  "d_w1": (wl.N, win, hid), "d_w2": (wl.N, hid, win)}
        self.grads = {}
        for n, s in shapes.items():
            if init is not None and n in init:
                self.grads[n] = torch.from_numpy(np.ascontiguousarray(init[n], np.float32)).to(dev)
            else:
                self.grads[n] = torch.full(s, float("nan"), dtype=torch.float32, device=dev)
        self.dx = torch.empty((wl.T, wl.d), dtype=self.out_dtype, device=dev)

    def backward(self):
        g = self.grads
        dcca = self.order == B.ORDER_DCCA
        B.bigmac_layer_backward(self.dims, self.params, self.x, self.dy, self.saved, self.dx,
                                g["d_w_down"] if dcca else None, g["d_w_up"] if dcca else None,
                                g["d_w_gate"], g["d_w1"], g["d_w2"], self.ws_train)

    def saved_views(self):
        """Routing arrays inside the saved block, as numpy."""
        lay = B.saved_layout(self.dims)
        wl = self.wl
        raw = self.saved.cpu().numpy()
        Tk = wl.T * wl.k
        f = lambda off, n, dt: raw[off:off + 4 * n].view(dt).copy()
        return {"topk_idx": f(lay["topk_idx"], Tk, np.int32).reshape(wl.T, wl.k),
                "topk_w": f(lay["topk_w"], Tk, np.float32).reshape(wl.T, wl.k),
                "expert_offsets": f(lay["expert_offsets"], wl.N + 1, np.int32),
                "slot_of": f(lay["slot_of"], Tk, np.int32).reshape(wl.T, wl.k)}

    def saved_aux(self):
        """(loss, share[N]) the training forward left in the saved block (dims.aux_alpha > 0)."""
        lay = B.saved_aux_layout(self.dims)
        raw = self.saved.cpu().numpy()
        loss = raw[lay["aux_loss"]:lay["aux_loss"] + 4].view(np.float32)[0]
        share = raw[lay["aux_share"]:lay["aux_share"] + 4 * self.wl.N].view(np.float32).copy()
        return float(loss), share


def add_cdac_weights(data: dict) -> dict:
    """The fine-grained layer with the same parameters: the BigMac expert matrices swapped
    (needs h == d): first matrix = W2 [N, d, r], second = W1 [N, r, d]."""
    out = dict(data)
    out["cdac_w1"] = data["w2"]
    out["cdac_w2"] = data["w1"]
    return out
