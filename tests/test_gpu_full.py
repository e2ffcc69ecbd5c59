"""Parity at the full sizes of the five workloads, in the launch configuration bench.py times.

The oracle cannot redo a whole workload in test time, so (module docstring of test_gpu_layer):
  * routing and permutation are compared in full, bit for bit;
  * y and dx are compared on sampled tokens (a token's y and dx depend on that token alone);
  * weight gradients of the dense-dy run are compared for chosen experts, for which the oracle
    is run on exactly the tokens routed to them (only those contribute to that expert's
    matrices and gating column);
  * all weight gradients are compared in a second GPU run whose dy is zero outside a token
    sample - the computation the oracle's token selection defines;
  * properties that hold at any size (rows of d_w_gate sum to zero, permutation invariants).
"""
import numpy as np
import pytest
import torch

from paper_2502_16927_amd import binding as B
from paper_2502_16927_amd import synth
from gpu_util import TOL, TOL_WIDE, DeviceLayer, add_cdac_weights, check_dx, check_weight_grads, host, rel_err, wgrad_err

pytestmark = pytest.mark.gpu


def routing_in_full(oracle, layer, data):
    wl = layer.wl
    v = layer.saved_views()
    idx, gate, _ = oracle.route(data["x"], data["w_gate"], data["gate_bias"], wl.k)
    off, slot, _ = oracle.permutation(idx, wl.N)
    assert np.array_equal(v["topk_idx"], idx), "top-k sets differ"
    assert np.array_equal(v["expert_offsets"], off) and np.array_equal(v["slot_of"], slot)
    assert np.abs(v["topk_w"] - gate).max() < 1e-6
    assert off[-1] == wl.T * wl.k and np.array_equal(np.sort(slot.ravel()), np.arange(wl.T * wl.k))
    return idx


def sample_tokens(T, n, seed):
    return np.sort(np.random.default_rng(seed).choice(T, size=min(n, T), replace=False)).astype(np.int32)


def bigmac_args(data):
    return (data["w_gate"], data["gate_bias"], data["w_down"], data["w_up"], data["w1"], data["w2"])


def run_training_workload(oracle, name, n_fwd, n_sel, experts_dense, flags=0, tol_y=TOL, sampled_scale=1.5, tol_w=TOL):
    wl = synth.WORKLOADS.get(name) or synth.NEXT_WORKLOADS[name]
    print(f"{name}: generating", flush=True)
    data = synth.generate(wl)
    layer = DeviceLayer(wl, data, flags=flags)
    y_inf = layer.forward(training=False).clone()
    y = layer.forward(training=True)
    torch.cuda.synchronize()
    assert torch.equal(y_inf, y)
    print(f"{name}: routing", flush=True)
    idx = routing_in_full(oracle, layer, data)
    counts = np.bincount(idx.ravel(), minlength=wl.N)
    sel = sample_tokens(wl.T, n_fwd, 1)
    ref_y = oracle.bigmac_forward(data["x"], *bigmac_args(data), wl.k, sel=sel)
    y_np = host(y)
    rms_y = float(np.sqrt(np.mean(ref_y ** 2)))
    e_y = np.abs(y_np[sel] - ref_y).max() / rms_y
    print(f"{name}: forward max-abs/rms on {len(sel)} tokens = {e_y:.4f}", flush=True)
    assert e_y < tol_y
    # dense dy: dx on the sampled tokens, weight gradients of chosen experts
    rng = np.random.default_rng(2)
    init = None
    if flags & B.FLAG_ACCUMULATE:      # running sums already in the buffers (fp32 accumulation into them)
        shapes = {"d_w_down": (wl.d, wl.r), "d_w_up": (wl.r, wl.d), "d_w_gate": (wl.d, wl.N),
                  "d_w1": (wl.N, wl.r, wl.h), "d_w2": (wl.N, wl.h, wl.r)}
        init = {n: (rng.standard_normal(s, dtype=np.float32) * np.float32(0.05)) for n, s in shapes.items()}
    layer.alloc_grads(init)
    layer.backward()
    torch.cuda.synchronize()
    g_dense = {n: host(v) - (init[n] if init else 0) for n, v in layer.grads.items()}
    dx_np = host(layer.dx)
    ref = oracle.bigmac_backward(data["x"], data["dy"], *bigmac_args(data), wl.k, sel=sel)
    e_dx = check_dx(dx_np[sel], ref["dx"][sel])
    print(f"{name}: dx on {len(sel)} tokens: worst token max-abs/rms = {e_dx[0]:.4f}, share of tokens above {TOL} = {e_dx[1]:.3%}", flush=True)
    scale = 1.5 if init else 1.0       # subtracting the initial sum costs fp32 round-off of the sum
    for e in experts_dense(counts):
        tok = np.nonzero((idx == e).any(axis=1))[0].astype(np.int32)
        ref_e = oracle.bigmac_backward(data["x"], data["dy"], *bigmac_args(data), wl.k, sel=tok)
        errs = {n: wgrad_err(g_dense[n][e], ref_e[n][e], len(tok)) for n in ("d_w1", "d_w2")}
        errs["d_w_gate"] = wgrad_err(g_dense["d_w_gate"][:, e], ref_e["d_w_gate"][:, e], len(tok))
        print(f"{name}: dense-dy gradients of expert {e} ({len(tok)} rows): {errs}", flush=True)
        assert all(v < tol_w * scale for v in errs.values()), errs
    gate_rows = np.abs(g_dense["d_w_gate"].sum(axis=1)).max() / np.abs(g_dense["d_w_gate"]).max()
    assert gate_rows < 2e-2, "rows of d_w_gate do not sum to zero"
    # sampled dy: every weight gradient against the oracle's token selection
    sel2 = sample_tokens(wl.T, n_sel, 3)
    masked = dict(data)
    masked["dy"] = np.zeros_like(data["dy"])
    masked["dy"][sel2] = data["dy"][sel2]
    layer.dy = B.to_device(masked["dy"], wl.dtype)
    layer.dims = B.dims_of(wl, flags=flags & ~B.FLAG_ACCUMULATE)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    ref2 = oracle.bigmac_backward(data["x"], data["dy"], *bigmac_args(data), wl.k, sel=sel2)
    cnt2 = np.bincount(idx[sel2].ravel(), minlength=wl.N)
    # a token sample leaves each expert a fraction of its rows: sums of fewer products have a
    # heavier-tailed error (module docstring of gpu_util.wgrad_err), hence the 1.5; the strict bar
    # is the dense-dy comparison above, on experts with all their rows
    worst = check_weight_grads({n: host(v) for n, v in layer.grads.items()}, ref2, cnt2, len(sel2), TOL, scale=sampled_scale)
    print(f"{name}: sampled-dy weight gradients ({len(sel2)} tokens): {worst}", flush=True)
    dx2 = host(layer.dx)
    check_dx(dx2[sel2], ref2["dx"][sel2])
    rest = np.setdiff1d(np.arange(wl.T), sel2)[:4096]
    assert not np.any(dx2[rest]), "dy = 0 must give dx = 0"


def test_gpt_medium_bigmac(oracle):
    run_training_workload(oracle, "gpt_medium", n_fwd=512, n_sel=4096, experts_dense=lambda c: [int(np.argmin(c)), int(np.argmax(c)), 17])


def test_gpt_medium_fine_grained_same_parameters(oracle):
    """The CDAC-order layer built from the same expert parameters (roles swapped), and the byte
    ratio of its permutes to BigMac's: r/d = 0.25 (the paper's -75 %, Table 4)."""
    wl = synth.WORKLOADS["gpt_medium"]
    data = add_cdac_weights(synth.generate(wl))
    layer = DeviceLayer(wl, data, order=B.ORDER_CDAC)
    y = layer.forward(training=True)
    torch.cuda.synchronize()
    idx = routing_in_full(oracle, layer, data)
    sel = sample_tokens(wl.T, 256, 1)
    ref_y = oracle.cdac_forward(data["x"], data["w_gate"], None, data["cdac_w1"], data["cdac_w2"], wl.k, sel=sel)
    assert np.abs(host(y)[sel] - ref_y).max() / np.sqrt(np.mean(ref_y ** 2)) < TOL
    sel2 = sample_tokens(wl.T, 4096, 3)
    dy = np.zeros_like(data["dy"])
    dy[sel2] = data["dy"][sel2]
    layer.dy = B.to_device(dy, wl.dtype)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    ref = oracle.cdac_backward(data["x"], data["dy"], data["w_gate"], None, data["cdac_w1"], data["cdac_w2"], wl.k, sel=sel2)
    check_dx(host(layer.dx)[sel2], ref["dx"][sel2])
    grads = {n: host(layer.grads[n]) for n in ("d_w_gate", "d_w1", "d_w2")}
    print(check_weight_grads(grads, ref, np.bincount(idx[sel2].ravel(), minlength=wl.N), len(sel2), TOL, dcca=False, scale=1.5), flush=True)
    assert B.permute_bytes(B.dims_of(wl)) / B.permute_bytes(B.dims_of(wl, B.ORDER_CDAC)) == wl.r / wl.d == 0.25


def test_vanilla_moe_structure(oracle):
    """The vanilla MoE layer (Fig. 2a: 8 full-width experts d -> 4d -> d, top-2) from the same
    kernels: CDAC order with the hidden width 4d."""
    wl = synth.NEXT_WORKLOADS["vanilla_moe"]
    data = add_cdac_weights(synth.generate(wl))
    layer = DeviceLayer(wl, data, order=B.ORDER_CDAC)
    y = layer.forward(training=True)
    torch.cuda.synchronize()
    idx = routing_in_full(oracle, layer, data)
    sel = sample_tokens(wl.T, 128, 1)
    ref_y = oracle.cdac_forward(data["x"], data["w_gate"], None, data["cdac_w1"], data["cdac_w2"], wl.k, sel=sel)
    err = np.abs(host(y)[sel] - ref_y).max() / np.sqrt(np.mean(ref_y ** 2))
    print(f"vanilla_moe: forward max-abs/rms = {err:.4f}", flush=True)
    assert err < TOL
    sel2 = sample_tokens(wl.T, 1024, 3)
    dy = np.zeros_like(data["dy"])
    dy[sel2] = data["dy"][sel2]
    layer.dy = B.to_device(dy, wl.dtype)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    ref = oracle.cdac_backward(data["x"], data["dy"], data["w_gate"], None, data["cdac_w1"], data["cdac_w2"], wl.k, sel=sel2)
    check_dx(host(layer.dx)[sel2], ref["dx"][sel2])
    grads = {n: host(layer.grads[n]) for n in ("d_w_gate", "d_w1", "d_w2")}
    print(check_weight_grads(grads, ref, np.bincount(idx[sel2].ravel(), minlength=wl.N), len(sel2), TOL, dcca=False, scale=1.5), flush=True)


def test_gpt_xl_accumulating_gradients(oracle):
    run_training_workload(oracle, "gpt_xl", n_fwd=256, n_sel=4096, experts_dense=lambda c: [int(np.argmin(c)), int(np.argmax(c))],
                          flags=B.FLAG_ACCUMULATE)


@pytest.mark.parametrize("name", ["gpt_2p7b", "gpt_6p7b"])
def test_larger_base_models(oracle, name):
    # the widths of the two larger models of the paper's training comparison (Fig. 3); small token
    # samples keep the oracle's share of the run short
    # Sampled dy: half the rows per expert (error of a sum relative to its size up by sqrt 2) and
    # the largest of 1e8-4e8 expert-gradient elements instead of gpt_medium's 2e7 (extreme value up
    # by ~1.1): 2 x the bar there; the strict bar is the dense-dy comparison on whole experts.
    run_training_workload(oracle, name, n_fwd=256, n_sel=4096, experts_dense=lambda c: [int(np.argmin(c)), int(np.argmax(c))],
                          tol_y=TOL_WIDE if name == "gpt_6p7b" else TOL, sampled_scale=2.0,
                          # d 4096, r 1024, h 4096 are the widest shapes (those of the decode workload): the
                          # storage floor that sets TOL_WIDE for y there carries over to the gradients built
                          # from the same bf16 tensors (measured 0.019-0.020 on whole experts)
                          tol_w=TOL_WIDE if name == "gpt_6p7b" else TOL)


@pytest.mark.parametrize("T", synth.DECODE_T_SWEEP)
def test_decode_sweep_forward(oracle, T):
    wl = synth.WORKLOADS["decode"].with_T(T)
    print(f"decode T={T}", flush=True)
    data = synth.generate(wl)
    layer = DeviceLayer(wl, data)
    y = host(layer.forward(training=False))
    torch.cuda.synchronize()
    sel = sample_tokens(T, 64, 1)
    ref = oracle.bigmac_forward(data["x"], *bigmac_args(data), wl.k, sel=sel)
    err = np.abs(y[sel] - ref).max() / np.sqrt(np.mean(ref ** 2))
    print(f"decode T={T}: max-abs/rms = {err:.4f}", flush=True)
    assert err < TOL_WIDE
    layer.forward(training=True)       # the routing arrays live in the saved block
    torch.cuda.synchronize()
    routing_in_full(oracle, layer, data)


def test_zipf_stress(oracle):
    def pick(counts):
        order = np.argsort(counts)
        return [int(order[0]), int(order[len(order) // 2])]      # the least loaded and a median expert
    run_training_workload(oracle, "zipf_stress", n_fwd=128, n_sel=768, experts_dense=pick, tol_y=TOL_WIDE)
