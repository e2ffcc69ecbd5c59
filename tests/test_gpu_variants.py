"""GPU parity of the two layer variants (expert biases, Table 3's 2rh term; router on x', the
alternative Section 3.1 names), of the activation itself over its whole range, and of a skewed
mid-size case whose weight gradients the oracle can redo in full."""
import numpy as np
import pytest
import torch

from paper_2502_16927_amd import binding as B
from paper_2502_16927_amd import synth
from gpu_util import (TOL, DeviceLayer, check_weight_grads, effective_rows, expert_effective_rows, few_rows_per_expert, host,
                      rel_err, rel_err_to_largest)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def with_biases(wl, data, seed=11, scale=0.05):
    """Biases of the size of the pre-activations' own spread (x' W1 has a standard deviation of 0.05 to 0.2 in
    these cases).  Much larger ones put a constant on every hidden unit that its bf16 rounding scales with while
    the weight gradients' RMS does not (measured with 0.3: d_w2 at 0.05 of its RMS from the rounding of H alone)."""
    rng = np.random.default_rng(seed)
    rnd = synth.round_to_bf16 if wl.dtype == B.BF16 else (lambda a: a)
    out = dict(data)
    out["b1"] = rnd((rng.standard_normal((wl.N, wl.h)) * scale).astype(np.float32))
    out["b2"] = rnd((rng.standard_normal((wl.N, wl.r)) * scale).astype(np.float32))
    return out


BIAS_CASES = [
    dict(T=96, d=128, r=64, N=8, k=2, h=128, dtype=B.BF16),
    dict(T=300, d=256, r=128, N=16, k=4, h=320, dtype=B.BF16),
    dict(T=130, d=128, r=64, N=8, k=3, h=192, dtype=B.F32, x_std=0.5),
    dict(T=257, d=192, r=64, N=24, k=8, h=192, dtype=B.BF16, zipf_s=1.2),
    dict(T=2560, d=512, r=512, N=16, k=8, h=2048, dtype=B.BF16),      # the 256-row tiles
]


@pytest.mark.parametrize("case", BIAS_CASES, ids=lambda c: "T{T}_d{d}_r{r}_N{N}_k{k}_h{h}_t{dtype}".format(**c))
@pytest.mark.parametrize("tiles", [0, B.FLAG_TILES_LARGE], ids=["tiles_auto", "tiles_large"])
def test_layer_with_expert_biases(oracle, case, tiles):
    if tiles and case["dtype"] != B.BF16:
        pytest.skip("the large tiles are a bf16 kernel")
    print("layer with expert biases", case, tiles, flush=True)
    wl = synth.small(**case)
    data = with_biases(wl, synth.generate(wl))
    layer = DeviceLayer(wl, data, flags=tiles)
    tol = TOL if wl.dtype == B.BF16 else 1e-4
    y_inf = host(layer.forward(training=False)).copy()
    y = host(layer.forward(training=True))
    torch.cuda.synchronize()
    args = (data["w_gate"], data["gate_bias"], data["w_down"], data["w_up"], data["w1"], data["w2"], wl.k)
    ref = oracle.bigmac_forward(data["x"], *args, b1=data["b1"], b2=data["b2"])
    assert np.array_equal(y_inf, y)
    assert rel_err(y, ref) < tol
    assert rel_err(y, oracle.bigmac_forward(data["x"], *args)) > 5 * tol, "the biases must matter in this case"
    g_ref = oracle.bigmac_backward(data["x"], data["dy"], *args, b1=data["b1"], b2=data["b2"])
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    assert rel_err(host(layer.dx), g_ref["dx"]) < tol, "dx"
    eff = expert_effective_rows(oracle, data, wl)
    grads = {n: host(v) for n, v in layer.grads.items()}
    print(check_weight_grads(grads, g_ref, eff, tol, few_rows=wl.dtype == B.BF16 and few_rows_per_expert(eff)), flush=True)
    # the bias gradients are plain column sums over an expert's rows: whole tensors against their RMS
    # (with a handful of rows per expert: against the largest element, like the other expert gradients)
    few = wl.dtype == B.BF16 and few_rows_per_expert(eff)
    for n in ("d_b1", "d_b2"):
        e = rel_err_to_largest(grads[n], g_ref[n]) if few else rel_err(grads[n], g_ref[n])
        print(n, round(e, 4), flush=True)
        assert e < tol, n
    # accumulate flag: added to what the buffers hold
    rng = np.random.default_rng(5)
    init = {n: rng.standard_normal(v.shape).astype(np.float32) * float(np.sqrt(np.mean(v * v)) + 1e-12) for n, v in g_ref.items() if n != "dx"}
    layer2 = DeviceLayer(wl, data, flags=B.FLAG_ACCUMULATE | tiles)
    layer2.forward(training=True)
    layer2.alloc_grads(init)
    layer2.backward()
    torch.cuda.synchronize()
    for n in ("d_b1", "d_b2"):
        g = host(layer2.grads[n]) - init[n]
        assert (rel_err_to_largest(g, g_ref[n]) if few else rel_err(g, g_ref[n])) < tol, n


def test_zero_biases_give_the_bits_of_no_biases():
    wl = synth.small(T=300, d=256, r=128, N=16, k=4, h=320)
    data = synth.generate(wl)
    zero = dict(data, b1=np.zeros((wl.N, wl.h), np.float32), b2=np.zeros((wl.N, wl.r), np.float32))
    a, b = DeviceLayer(wl, data), DeviceLayer(wl, zero)
    ya, yb = a.forward(training=True), b.forward(training=True)
    a.alloc_grads(); b.alloc_grads()
    a.backward(); b.backward()
    torch.cuda.synchronize()
    assert torch.equal(ya, yb) and torch.equal(a.dx, b.dx)
    for n in a.grads:
        assert torch.equal(a.grads[n], b.grads[n]), n


@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_grouped_ffn_with_biases(oracle, dtype):
    T, r, h, N, k, d = 500, 128, 192, 8, 4, 256
    rng = np.random.default_rng(3)
    rnd = synth.round_to_bf16 if dtype == B.BF16 else (lambda a: a)
    idx_np = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    off_np, _, _ = oracle.permutation(idx_np, N)
    xp = rnd(rng.standard_normal((T * k, r)).astype(np.float32))
    w1 = rnd((rng.standard_normal((N, r, h)) * 0.1).astype(np.float32))
    w2 = rnd((rng.standard_normal((N, h, r)) * 0.1).astype(np.float32))
    b1 = rnd((rng.standard_normal((N, h)) * 0.5).astype(np.float32))
    b2 = rnd((rng.standard_normal((N, r)) * 0.5).astype(np.float32))
    dims = B.make_dims(T, d, r, N, k, h, dtype)
    o = torch.empty((T * k, r), dtype=B.act_dtype(dtype), device=DEV)
    a = torch.empty((T * k, h), dtype=B.act_dtype(dtype), device=DEV)
    ws = B.alloc_bytes(B.workspace_bytes(dims, B.WS_GROUPED_FFN))
    B.bigmac_grouped_ffn(dims, B.to_device(xp, dtype), torch.from_numpy(off_np).to(DEV), B.to_device(w1, dtype), B.to_device(w2, dtype),
                         a, o, ws, b1=B.to_device(b1, dtype), b2=B.to_device(b2, dtype))
    torch.cuda.synchronize()
    ref_o, ref_a = oracle.expert_rows(xp, off_np, w1, w2, want_a=True, b1=b1, b2=b2)
    tol = TOL if dtype == B.BF16 else 1e-4
    assert rel_err(host(a), ref_a) < tol and rel_err(host(o), ref_o) < tol


@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_activation_over_its_range(oracle, dtype):
    """The GPU's GELU (its own polynomial evaluation) against the oracle's erf form over
    a in [-6, 6]: one expert whose two matrices are the identity and the argument fed in as x_perm,
    so that o = gelu(a) element by element (rounded once to the storage type)."""
    r = h = 64
    T = 4096
    grid = np.linspace(-6.0, 6.0, T * r, dtype=np.float64).reshape(T, r).astype(np.float32)
    rnd = synth.round_to_bf16 if dtype == B.BF16 else (lambda a: a)
    xp = rnd(grid)
    eye = np.eye(r, dtype=np.float32)[None]
    off = np.array([0, T], np.int32)
    dims = B.make_dims(T, 64, r, 1, 1, h, dtype)
    o = torch.empty((T, r), dtype=B.act_dtype(dtype), device=DEV)
    a = torch.empty((T, h), dtype=B.act_dtype(dtype), device=DEV)
    ws = B.alloc_bytes(B.workspace_bytes(dims, B.WS_GROUPED_FFN))
    B.bigmac_grouped_ffn(dims, B.to_device(xp, dtype), torch.from_numpy(off).to(DEV), B.to_device(eye, dtype), B.to_device(eye, dtype), a, o, ws)
    torch.cuda.synchronize()
    ref_o, ref_a = oracle.expert_rows(xp, off, eye, eye, want_a=True)
    assert np.array_equal(host(a), ref_a.astype(np.float32))                 # the pre-activation is the argument itself
    err = np.abs(host(o).astype(np.float64) - ref_o)
    if dtype == B.F32:
        assert err.max() < 1e-6, err.max()                                   # the fp32 path's polynomial: < 4e-7 absolute
    else:
        # bf16 result: half a unit in the last place of the result (up to 2^-8 relative) plus the evaluation's own 3e-5 relative
        # (and 4e-7 absolute: the far negative tail, where the result itself is below 1e-6)
        assert np.all(err <= np.abs(ref_o) * (2.0 ** -8 + 1e-4) + 4e-7), float((err - np.abs(ref_o) * (2.0 ** -8 + 1e-4)).max())


def test_activation_derivative_over_its_range(oracle):
    """GELU' through the layer's backward pass, read off dx of a layer whose pre-activation sweeps
    [-6, 6]: x' = x (W_down = I), a = x' (W1 = I), o = gelu(a) (W2 = I), y = o (W_up = I), dy = 1
    =>  dx = gelu'(a) element by element (top-1 routing: the gate value is 1)."""
    d = r = h = 64
    T = 2048
    wl = synth.small(T=T, d=d, r=r, N=8, k=1, h=h)
    a = synth.round_to_bf16(np.linspace(-6.0, 6.0, T * d, dtype=np.float64).reshape(T, d).astype(np.float32))
    eye = np.eye(d, dtype=np.float32)
    data = {"x": a, "dy": np.ones((T, d), np.float32), "w_gate": np.zeros((d, 8), np.float32), "gate_bias": None,
            "w_down": eye, "w_up": eye, "w1": np.tile(eye[None], (8, 1, 1)), "w2": np.tile(eye[None], (8, 1, 1))}
    layer = DeviceLayer(wl, data)
    layer.forward(training=True)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    ref = oracle.bigmac_backward(data["x"], data["dy"], data["w_gate"], None, eye, eye, data["w1"], data["w2"], 1)["dx"]
    # zero router weights: every token goes to expert 0 with gate 1 and no gate gradient reaches dx
    err = np.abs(host(layer.dx).astype(np.float64) - ref)
    # dA = dO * gelu'(A) is rounded to bf16 (2^-9 relative), gelu' itself is within 4e-5 absolute of the erf form
    assert np.all(err <= np.abs(ref) * 2.0 ** -8 + 1e-4), float(err.max())


# ------------------------------------------------------------------ router on x' ----------------------

def exact_low_inputs(wl, seed=21):
    """Inputs whose x' = x W_down is exact in every arithmetic: x in {-1, 0, 1}, W_down in {-1, 0, 1} / 16
    with few non-zeros per column, so that x' is a small multiple of 1/16 that bf16 holds exactly.  The
    router of the GPU path and the oracle's then read the very same x', and the routing can be
    compared bit for bit although x' is a computed quantity."""
    rng = np.random.default_rng(seed)
    data = synth.generate(wl)
    data["x"] = rng.integers(-1, 2, size=(wl.T, wl.d)).astype(np.float32)
    wd = np.zeros((wl.d, wl.r), np.float32)
    for c in range(wl.r):
        rows = rng.choice(wl.d, size=24, replace=False)
        wd[rows, c] = rng.choice([-1.0, 1.0], size=24) / 16.0
    data["w_down"] = wd
    data["w_gate"] = (rng.standard_normal((wl.r, wl.N)) * 0.3).astype(np.float32)
    return data


@pytest.mark.parametrize("case", [dict(T=300, d=256, r=128, N=16, k=4, h=192, dtype=B.BF16), dict(T=130, d=128, r=64, N=8, k=3, h=128, dtype=B.F32),
                                  dict(T=64, d=256, r=256, N=8, k=2, h=64, dtype=B.BF16)],
                         ids=lambda c: "T{T}_d{d}_r{r}_N{N}_k{k}_t{dtype}".format(**c))
def test_router_on_low_exact_inputs(oracle, case):
    print("router on x', exact x'", case, flush=True)
    wl = synth.small(**case)
    data = exact_low_inputs(wl)
    mode = oracle.ROUTE_LOW_BF16 if wl.dtype == B.BF16 else oracle.ROUTE_LOW_F32
    xl = oracle.stored_low(data["x"], data["w_down"], mode)
    assert np.array_equal(xl, (data["x"].astype(np.float64) @ data["w_down"].astype(np.float64)).astype(np.float32)), "x' must be exact"
    layer = DeviceLayer(wl, data, flags=B.FLAG_ROUTE_LOW)
    tol = TOL if wl.dtype == B.BF16 else 1e-4
    y_inf = host(layer.forward(training=False)).copy()
    y = host(layer.forward(training=True))
    torch.cuda.synchronize()
    idx, gate, _, _ = oracle.route_low(data["x"], data["w_down"], data["w_gate"], None, wl.k, mode=mode)
    off, slot, _ = oracle.permutation(idx, wl.N)
    v = layer.saved_views()
    assert np.array_equal(v["topk_idx"], idx), "top-k sets differ"
    assert np.array_equal(v["expert_offsets"], off) and np.array_equal(v["slot_of"], slot)
    assert np.abs(v["topk_w"] - gate).max() < 1e-6
    args = (data["w_gate"], None, data["w_down"], data["w_up"], data["w1"], data["w2"], wl.k)
    ref = oracle.bigmac_forward(data["x"], *args, route_low=mode)
    assert np.array_equal(y_inf, y) and rel_err(y, ref) < tol
    g_ref = oracle.bigmac_backward(data["x"], data["dy"], *args, route_low=mode)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    assert rel_err(host(layer.dx), g_ref["dx"]) < tol, "dx"
    eff = effective_rows(idx, gate, wl.N)
    grads = {n: host(t) for n, t in layer.grads.items()}
    assert grads["d_w_gate"].shape == (wl.r, wl.N)
    print(check_weight_grads(grads, g_ref, eff, tol, few_rows=wl.dtype == B.BF16 and few_rows_per_expert(eff)), flush=True)


def test_router_on_low_random_inputs(oracle):
    """Ordinary inputs: the GPU's x' (fp32 accumulation in MFMA order, rounded to bf16) and the
    oracle's (fp64, rounded) differ in the last bit of a few elements, so a token whose k-th and
    (k+1)-th logits are closer than that may be routed differently.  Compared: the tokens whose
    decision margin in the oracle exceeds the largest logit change one bf16 unit of x' can cause
    must be routed identically, and they are nearly all; y and dx are compared on those tokens."""
    wl = synth.small(T=2000, d=512, r=128, N=16, k=4, h=256)
    data = synth.generate(wl)
    rng = np.random.default_rng(4)
    data["w_gate"] = (rng.standard_normal((wl.r, wl.N)) * 0.1).astype(np.float32)
    layer = DeviceLayer(wl, data, flags=B.FLAG_ROUTE_LOW)
    y = host(layer.forward(training=True))
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    idx, gate, logits, xl = oracle.route_low(data["x"], data["w_down"], data["w_gate"], None, wl.k, mode=oracle.ROUTE_LOW_BF16)
    srt = np.sort(logits.astype(np.float64), axis=1)[:, ::-1]
    gaps = np.abs(np.diff(srt[:, :wl.k + 1], axis=1)).min(axis=1)          # smallest gap among the picks and to the first non-pick
    # one element of x' off by one bf16 unit (at most 2^-7 relative) moves a logit by at most |x'| 2^-7 max|w_gate|;
    # allow two such elements per token, and both logits of a pair to move
    bound = 2 * np.abs(xl).max(axis=1) * 2.0 ** -7 * np.abs(data["w_gate"]).max()
    safe = gaps > 2 * bound
    assert safe.mean() > 0.2, safe.mean()
    v = layer.saved_views()
    assert np.array_equal(v["topk_idx"][safe], idx[safe])
    same = np.all(v["topk_idx"] == idx, axis=1)
    print(f"router on x': {same.mean():.4f} of the tokens routed as the oracle routes them, {safe.mean():.4f} provably", flush=True)
    assert same.mean() > 0.98
    args = (data["w_gate"], None, data["w_down"], data["w_up"], data["w1"], data["w2"], wl.k)
    sel = np.flatnonzero(same).astype(np.int32)
    ref = oracle.bigmac_forward(data["x"], *args, route_low=oracle.ROUTE_LOW_BF16, sel=sel)
    assert rel_err(y[sel], ref) < TOL
    g_ref = oracle.bigmac_backward(data["x"], data["dy"], *args, route_low=oracle.ROUTE_LOW_BF16, sel=sel)
    assert rel_err(host(layer.dx)[sel], g_ref["dx"][sel]) < TOL


def test_route_call_on_low_width_input(oracle):
    """The router call itself on an r-wide input (what the layer does with the flag): bit-exact."""
    T, r, N, k = 700, 192, 24, 5
    rng = np.random.default_rng(8)
    xl = synth.round_to_bf16(rng.standard_normal((T, r)).astype(np.float32))
    wg = (rng.standard_normal((r, N)) * 0.2).astype(np.float32)
    dims = B.make_dims(T, r, 64, N, k, 64)
    idx = torch.empty((T, k), dtype=torch.int32, device=DEV)
    w = torch.empty((T, k), dtype=torch.float32, device=DEV)
    lg = torch.empty((T, N), dtype=torch.float32, device=DEV)
    B.bigmac_route(dims, B.to_device(xl, B.BF16), B.to_device(wg, B.F32), None, idx, w, lg)
    torch.cuda.synchronize()
    r_idx, r_gate, r_logits = oracle.route(xl, wg, None, k)
    assert np.array_equal(host(lg).view(np.uint32), r_logits.view(np.uint32))
    assert np.array_equal(host(idx), r_idx) and np.abs(host(w) - r_gate).max() < 1e-6


# ------------------------------------------------------------------ skewed mid-size case -----------------

def test_skewed_mid_size_all_weight_gradients(oracle):
    """Strongly skewed routing at a size the oracle redoes in full: one expert holds most of the
    16 k tokens (a long ragged K in the weight-gradient products, cut at equal cost over the XCDs,
    and many row tiles of one expert), others a handful.  Dense dy; every expert's blocks with
    enough rows against their own RMS, the shared gradients as whole tensors."""
    wl = synth.small(T=16384, d=256, r=128, N=8, k=2, h=256, zipf_s=3.0)
    data = synth.generate(wl)
    layer = DeviceLayer(wl, data)
    y = host(layer.forward(training=True))
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    idx, gate, _ = oracle.route(data["x"], data["w_gate"], data["gate_bias"], wl.k)
    counts = np.bincount(idx.ravel(), minlength=wl.N)
    print("rows per expert", counts, flush=True)
    assert counts.max() > 8192 and counts.min() < 1024
    v = layer.saved_views()
    assert np.array_equal(v["topk_idx"], idx)
    args = (data["w_gate"], data["gate_bias"], data["w_down"], data["w_up"], data["w1"], data["w2"], wl.k)
    assert rel_err(y, oracle.bigmac_forward(data["x"], *args)) < TOL
    g_ref = oracle.bigmac_backward(data["x"], data["dy"], *args)
    assert rel_err(host(layer.dx), g_ref["dx"]) < TOL
    eff = effective_rows(idx, gate, wl.N)
    print("effective rows", np.round(eff), flush=True)
    print(check_weight_grads({n: host(t) for n, t in layer.grads.items()}, g_ref, eff, TOL, skewed=True), flush=True)


def _ragged_k_regime(counts: np.ndarray) -> str:
    """Which schedule the weight-gradient products take for these rows per expert, restated from
    the builder's rule: a group costs its 32-row k tiles + 8; eight equal runs of groups are kept
    while the fullest stays within 9/8 of the even share; else whole groups are dealt to the XCDs
    largest first if the fullest XCD then stays within 1.2 of the share; else a cut of equal cost
    that splits groups."""
    cost = (counts + 31) // 32 + 8
    total, n = int(cost.sum()), len(counts)
    incl = np.cumsum(cost)

    def before(q):
        gi = q >> 16
        return total if gi >= n else int(incl[gi] - cost[gi]) + (((q & 0xFFFF) * int(cost[gi])) >> 16)

    worst = max(before((n * (x + 1) << 16) // 8) - before((n * x << 16) // 8) for x in range(8))
    if worst * 64 <= total * 9:
        return "equal runs"
    load = [0] * 8
    for g in sorted(range(n), key=lambda g: (-cost[g], g)):
        b = min(range(8), key=lambda x: (load[x], x))
        load[b] += int(cost[g])
    return "whole groups" if max(load) * 40 <= total * 6 else "split groups"


@pytest.mark.parametrize("T,regime", [(8192, "whole groups"), (16384, "split groups")])
def test_skewed_many_experts_all_weight_gradients(oracle, T, regime):
    """128 experts under Zipf routing at sizes the oracle redoes in full: more groups than one
    wavefront holds (the tile maps come from the workgroup-wide builder) and both schedules of the
    skewed ragged-K products, each group's gradient block checked against the oracle."""
    wl = synth.small(T=T, d=128, r=64, N=128, k=4, h=128, zipf_s=1.2)
    data = synth.generate(wl)
    idx, gate, _ = oracle.route(data["x"], data["w_gate"], data["gate_bias"], wl.k)
    counts = np.bincount(idx.ravel(), minlength=wl.N)
    assert _ragged_k_regime(counts) == regime
    layer = DeviceLayer(wl, data)
    y = host(layer.forward(training=True))
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    v = layer.saved_views()
    assert np.array_equal(v["topk_idx"], idx)
    r_off, r_slot, _ = oracle.permutation(idx, wl.N)
    assert np.array_equal(v["expert_offsets"], r_off) and np.array_equal(v["slot_of"], r_slot)
    args = (data["w_gate"], data["gate_bias"], data["w_down"], data["w_up"], data["w1"], data["w2"], wl.k)
    assert rel_err(y, oracle.bigmac_forward(data["x"], *args)) < TOL
    g_ref = oracle.bigmac_backward(data["x"], data["dy"], *args)
    assert rel_err(host(layer.dx), g_ref["dx"]) < TOL
    eff = effective_rows(idx, gate, wl.N)
    print(check_weight_grads({n: host(t) for n, t in layer.grads.items()}, g_ref, eff, TOL, skewed=True), flush=True)
