"""Parity of the whole layer (forward and backward, both orders) against the CPU oracle.

Small workloads are compared element by element.  The full-size workloads run in the launch
configuration the benchmark times; there the routing and permutation are still compared in full
(the oracle's routing is cheap), outputs and dx on sampled tokens, and the weight gradients
through a dy that is zero outside the sampled tokens (exactly what the oracle's token selection
computes), plus properties that hold at any size."""
import numpy as np
import pytest
import torch

from paper_2502_16927_amd import binding as B
from paper_2502_16927_amd import synth
from gpu_util import TOL, DeviceLayer, add_cdac_weights, check_weight_grads, expert_effective_rows, few_rows_per_expert, host, rel_err

pytestmark = pytest.mark.gpu

SMALL = [
    dict(T=96, d=128, r=64, N=8, k=2, h=128, dtype=B.BF16),
    dict(T=300, d=256, r=128, N=16, k=4, h=320, dtype=B.BF16),
    dict(T=1500, d=256, r=128, N=8, k=2, h=256, dtype=B.BF16),
    dict(T=257, d=192, r=64, N=24, k=8, h=192, dtype=B.BF16, zipf_s=1.2),
    dict(T=64, d=64, r=64, N=8, k=8, h=64, dtype=B.BF16),
    dict(T=1, d=64, r=64, N=8, k=1, h=64, dtype=B.BF16),
    dict(T=200, d=768, r=256, N=8, k=2, h=128, dtype=B.BF16),   # few tiles, long K: the shared projections split K
    dict(T=130, d=128, r=64, N=8, k=3, h=192, dtype=B.F32, x_std=0.5),
    # enough rows, tiles and K for the 256-row workgroup tiles in expert-up and the GELU' product
    # (not in expert-down and its counterpart, which have 4 column tiles): both tile maps in one step
    dict(T=2560, d=512, r=512, N=16, k=8, h=2048, dtype=B.BF16),
    # the same with a hidden width that ends inside a 256-column tile (expert-up's 128 x 256 tiles)
    dict(T=2560, d=512, r=512, N=16, k=8, h=1984, dtype=B.BF16, zipf_s=0.8),
    # the router's share of dx: 65..128 experts (narrower LDS tile), N % 4 != 0 (scalar tile fill),
    # k = 8 + 4 + 1 picks, k = 64 (staging limit), d not a multiple of the tile width, and more than
    # 128 experts (per-token kernel on a transposed copy of the router weights)
    dict(T=300, d=192, r=64, N=96, k=5, h=64, dtype=B.BF16),
    dict(T=130, d=128, r=64, N=6, k=3, h=64, dtype=B.F32, x_std=0.5),
    dict(T=200, d=320, r=64, N=64, k=13, h=64, dtype=B.BF16),
    dict(T=70, d=128, r=64, N=128, k=64, h=64, dtype=B.BF16),
    dict(T=90, d=128, r=64, N=200, k=4, h=64, dtype=B.BF16),
    # 128 tiles under K = 576: descend and the data gradient of ascend take the 128 x 64 tile with
    # 64-deep k tiles (ragged last row tile, 7 column tiles; r is always a multiple of 64 here)
    dict(T=4000, d=576, r=448, N=8, k=2, h=64, dtype=B.BF16),
]


def oracle_forward(oracle, data, k, sel=None):
    return oracle.bigmac_forward(data["x"], data["w_gate"], data["gate_bias"], data["w_down"], data["w_up"],
                                 data["w1"], data["w2"], k, sel=sel)


def check_routing(oracle, layer, data):
    wl = layer.wl
    v = layer.saved_views()
    idx, gate, _ = oracle.route(data["x"], data["w_gate"], data["gate_bias"], wl.k)
    off, slot, _ = oracle.permutation(idx, wl.N)
    assert np.array_equal(v["topk_idx"], idx), "top-k sets differ"
    assert np.array_equal(v["expert_offsets"], off)
    assert np.array_equal(v["slot_of"], slot)
    assert np.abs(v["topk_w"] - gate).max() < 1e-6
    return idx


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "T{T}_d{d}_r{r}_N{N}_k{k}_h{h}_t{dtype}".format(**c))
def test_small_forward_backward(oracle, case):
    print("small layer", case, flush=True)
    wl = synth.small(**case)
    data = synth.generate(wl)
    layer = DeviceLayer(wl, data)
    tol = TOL if wl.dtype == B.BF16 else 1e-4
    y_inf = host(layer.forward(training=False)).copy()
    y = host(layer.forward(training=True))
    torch.cuda.synchronize()
    ref = oracle_forward(oracle, data, wl.k)
    assert np.array_equal(y_inf, y), "inference and training forward differ"
    assert rel_err(y, ref) < tol
    idx = check_routing(oracle, layer, data)
    counts = expert_effective_rows(oracle, data, wl)
    g_ref = oracle.bigmac_backward(data["x"], data["dy"], data["w_gate"], data["gate_bias"], data["w_down"],
                                   data["w_up"], data["w1"], data["w2"], wl.k)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    assert rel_err(host(layer.dx), g_ref["dx"]) < tol, "dx"
    print(check_weight_grads({n: host(v) for n, v in layer.grads.items()}, g_ref, counts, tol, few_rows=wl.dtype == B.BF16 and few_rows_per_expert(counts)), flush=True)
    # accumulate flag: gradients are added to what the buffers hold
    rng = np.random.default_rng(5)
    init = {n: rng.standard_normal(v.shape).astype(np.float32) * float(np.sqrt(np.mean(v * v)) + 1e-12)
            for n, v in g_ref.items() if n != "dx"}
    layer2 = DeviceLayer(wl, data, flags=B.FLAG_ACCUMULATE)
    layer2.forward(training=True)
    layer2.alloc_grads(init)
    layer2.backward()
    torch.cuda.synchronize()
    check_weight_grads({n: host(v) - init[n] for n, v in layer2.grads.items()}, g_ref, counts, tol, few_rows=wl.dtype == B.BF16 and few_rows_per_expert(counts))


@pytest.mark.parametrize("case", [SMALL[1], SMALL[3], SMALL[5], SMALL[8], SMALL[9], dict(T=700, d=128, r=192, N=8, k=2, h=448, dtype=B.BF16)],
                         ids=lambda c: "T{T}_d{d}_r{r}_N{N}_k{k}_h{h}".format(**c))
def test_large_tiles_give_the_same_bits(case):
    """The 256 x 256 workgroup tiles add the same products in the same order as the smaller ones:
    forcing them on (ragged tails, widths that are no multiple of 256, empty experts, T = 1) and
    forbidding them must give identical outputs and gradients."""
    print("large tiles", case, flush=True)
    wl = synth.small(**case)
    data = synth.generate(wl)
    outs = []
    for flag in (B.FLAG_TILES_SMALL, B.FLAG_TILES_LARGE):
        layer = DeviceLayer(wl, data, flags=flag)
        layer.forward(training=True)
        layer.alloc_grads()
        layer.backward()
        torch.cuda.synchronize()
        outs.append([layer.y.clone(), layer.dx.clone()] + [layer.grads[n].clone() for n in sorted(layer.grads)])
    for u, v in zip(*outs):
        assert torch.equal(u, v)


@pytest.mark.parametrize("order", [B.ORDER_DCCA, B.ORDER_CDAC])
@pytest.mark.parametrize("tiles", [0, B.FLAG_TILES_LARGE])
def test_dispatch_folded_into_the_expert_product(order, tiles):
    """A forward-only call reads the rows of the expert-up product from x' (x in the fine-grained
    order) through src_of instead of dispatching them first.  Same bits as with the dispatch
    (BIGMAC_FLAG_NO_FUSED_DISPATCH) and as the training forward: ragged and empty experts,
    a capacity that drops pairs, every tile shape."""
    wl = synth.small(T=1100, d=256, r=128, N=24, k=4, h=256, zipf_s=1.5)
    data = synth.generate(wl)
    if order == B.ORDER_CDAC:
        data = add_cdac_weights(data)
    for capacity in (0, B.expert_capacity(wl.T, wl.k, wl.N, 0.7)):
        outs = []
        for flags, training in ((tiles, False), (tiles | B.FLAG_NO_FUSED_DISPATCH, False), (tiles, True)):
            layer = DeviceLayer(wl, data, order=order, flags=flags, capacity=capacity)
            outs.append(host(layer.forward(training=training)).copy())
        assert np.isfinite(outs[0]).all() and np.abs(outs[0]).max() > 0
        assert np.array_equal(outs[0], outs[1]), "folded dispatch differs from the dispatched forward"
        assert np.array_equal(outs[0], outs[2]), "inference differs from the training forward"


@pytest.mark.parametrize("case", [dict(T=1100, d=256, r=128, N=24, k=4, h=256, zipf_s=1.5), dict(T=200, d=320, r=64, N=64, k=13, h=64),
                                  dict(T=1, d=64, r=64, N=8, k=1, h=64), dict(T=4000, d=576, r=448, N=8, k=2, h=64),
                                  dict(T=200, d=768, r=256, N=8, k=2, h=128)],
                         ids=lambda c: "T{T}_d{d}_r{r}_N{N}_k{k}_h{h}".format(**c))
def test_dispatch_folded_into_the_descending_projection(case):
    """A training forward has the descending projection write x' straight into the permuted copy
    (one store per pick, dropped pairs none).  Same bits as with the copy kernel
    (BIGMAC_FLAG_NO_FUSED_DISPATCH) in y, dx and every weight gradient (dW1 contracts over all rows
    of the permuted copy): more picks than one pass of the epilogue takes, a capacity that drops
    pairs, T = 1, a shape whose projection runs on its 128 x 64 tile, and one summed from K slices (not folded)."""
    wl = synth.small(**case)
    data = synth.generate(wl)
    for capacity in (0, B.expert_capacity(wl.T, wl.k, wl.N, 0.7)):
        outs = []
        for flags in (0, B.FLAG_NO_FUSED_DISPATCH):
            layer = DeviceLayer(wl, data, flags=flags, capacity=capacity)
            layer.forward(training=True)
            layer.alloc_grads()
            layer.backward()
            torch.cuda.synchronize()
            outs.append([layer.y.clone(), layer.dx.clone()] + [layer.grads[n].clone() for n in sorted(layer.grads)])
        assert torch.isfinite(outs[0][0]).all() and outs[0][0].abs().max() > 0
        for u, v in zip(*outs):
            assert torch.equal(u, v)


def test_variants_agree_bit_for_bit_on_random_shapes():
    """Tile shape, tile order in time and the folded dispatch (rows read through the index by the
    expert-up product, or written through it by the descending projection) only change who
    computes what and where the rows travel, never the arithmetic: on seeded random shapes (single
    experts, k = N, T = 1, skewed and capacity-clipped routing) every variant gives the bits of the
    plain training step, gradients included (dW1 contracts over every row of the permuted copy)."""
    rng = np.random.default_rng(11)
    for it in range(16):
        d, r = int(rng.choice([64, 128, 192, 256, 512])), int(rng.choice([64, 128, 192, 256, 512]))
        h = int(rng.choice([64, 128, 320, 512, 1024, 2048]))
        N = int(rng.choice([1, 2, 3, 8, 16, 24, 64]))
        k = int(rng.integers(1, min(N, 8) + 1))
        T = int(rng.choice([1, 7, 100, 257, 1000, 2500, 4097]))
        case = dict(T=T, d=d, r=r, N=N, k=k, h=h, zipf_s=float(rng.choice([0.0, 1.2, 3.0])))
        capacity = B.expert_capacity(T, k, N, 0.8) if rng.random() < 0.3 else 0
        print("random shape", it, case, "capacity", capacity, flush=True)
        wl = synth.small(**case)
        data = synth.generate(wl)
        ref = None
        for flags, training in ((B.FLAG_NO_FUSED_DISPATCH, True), (0, True), (0, False), (B.FLAG_NO_FUSED_DISPATCH, False),
                                (B.FLAG_TILES_LARGE, False), (B.FLAG_TILES_LARGE, True), (B.FLAG_TILES_SMALL, True)):
            layer = DeviceLayer(wl, data, flags=flags, capacity=capacity)
            out = {"y": host(layer.forward(training=training)).copy()}
            if training and N % 8 == 0:
                layer.alloc_grads()
                layer.backward()
                torch.cuda.synchronize()
                out.update({n: host(g).copy() for n, g in layer.grads.items()}, dx=host(layer.dx).copy())
            if ref is None:
                ref = out
                assert np.isfinite(ref["y"]).all()
            for n in out:
                if n in ref:
                    assert np.array_equal(ref[n], out[n]), (n, case, flags, training)


def test_variants_agree_bit_for_bit_on_mid_size_shapes():
    """The same at sizes where the tile policy leaves the square tile (128 x 256 and 256 x 256 tiles,
    64-deep k tiles, 128 experts with whole-group weight-gradient schedules, hidden widths that end
    inside a column tile): every variant gives the bits of the step that forbids the large tiles
    and dispatches with the copy kernel, gradients included."""
    rng = np.random.default_rng(5)
    for it in range(8):
        d, r = int(rng.choice([512, 1024, 2048])), int(rng.choice([512, 1024]))
        h = int(rng.choice([1024, 1984, 2048, 2304]))
        N, k, T = int(rng.choice([8, 16, 72, 128])), int(rng.choice([2, 4, 8])), int(rng.choice([2560, 6000, 8192, 12000]))
        case = dict(T=T, d=d, r=r, N=N, k=k, h=h, zipf_s=float(rng.choice([0.0, 0.8, 1.2])))
        capacity = B.expert_capacity(T, k, N, 0.8) if rng.random() < 0.25 else 0
        print("mid-size shape", it, case, "capacity", capacity, flush=True)
        wl = synth.small(**case)
        data = synth.generate(wl)
        ref = None
        for flags, training in ((B.FLAG_NO_FUSED_DISPATCH | B.FLAG_TILES_SMALL, True), (0, True), (B.FLAG_TILES_LARGE, True), (0, False)):
            layer = DeviceLayer(wl, data, flags=flags, capacity=capacity)
            out = {"y": host(layer.forward(training=training)).copy()}
            if training:
                layer.alloc_grads()
                layer.backward()
                torch.cuda.synchronize()
                out.update({n: host(g).copy() for n, g in layer.grads.items()}, dx=host(layer.dx).copy())
            del layer
            if ref is None:
                ref = out
                assert np.isfinite(ref["y"]).all() and np.abs(ref["y"]).max() > 0
            for n in out:
                assert np.array_equal(ref[n], out[n]), (n, case, flags, training)


def test_all_bf16_wire_format(oracle):
    """BIGMAC_FLAG_WIRE_BF16 (Table 4's BF16 transfers taken literally: expert outputs and the gradient
    of the dispatched rows rounded to bf16 between the expert products and the combine kernels):
    same routing, same saved activations; y, dx and the gradients stay at the bar on this shape
    and within a bf16 rounding's reach of the default (fp32) wire format."""
    wl = synth.small(T=1024, d=256, r=128, N=8, k=2, h=256)
    data = synth.generate(wl)
    ref_y = oracle_forward(oracle, data, wl.k)
    outs = []
    for flags in (0, B.FLAG_WIRE_BF16):
        layer = DeviceLayer(wl, data, flags=flags)
        y = layer.forward(training=True)
        layer.alloc_grads()
        layer.backward()
        torch.cuda.synchronize()
        outs.append({"y": host(y), "dx": host(layer.dx), **{n: host(g) for n, g in layer.grads.items()}})
    a, b = outs
    assert rel_err(a["y"], ref_y) < TOL and rel_err(b["y"], ref_y) < TOL, (rel_err(a["y"], ref_y), rel_err(b["y"], ref_y))
    worst = {}
    for n in a:
        if n in ("y", "dx", "d_w_gate"):                                # what sees O or dx_perm: the flag changes it ...
            assert not np.array_equal(a[n], b[n]), n
        if n in ("d_w1", "d_w2"):                                       # (the expert products' own operands are bf16 either way)
            assert np.array_equal(a[n], b[n]), n
        worst[n] = rel_err(b[n], a[n])
        assert worst[n] < TOL, (n, worst[n])                            # ... by no more than a few bf16 roundings
    print("all-bf16 wire format against the default: max-abs/rms", {n: round(v, 4) for n, v in worst.items()}, flush=True)


def test_bf16_output_is_the_rounded_fp32_output(oracle):
    wl = synth.small(T=200, d=128, r=64, N=8, k=2, h=128)
    data = synth.generate(wl)
    a = DeviceLayer(wl, data)
    b = DeviceLayer(wl, data, flags=B.FLAG_OUT_BF16)
    ya, yb = a.forward(training=True), b.forward(training=True)
    assert torch.equal(ya.to(torch.bfloat16), yb)
    a.alloc_grads(); b.alloc_grads()
    a.backward(); b.backward()
    torch.cuda.synchronize()
    assert torch.equal(a.dx.to(torch.bfloat16), b.dx)
    for n in a.grads:
        assert torch.equal(a.grads[n], b.grads[n])


def test_gather_probe_runs_and_rejects_bad_sizes():
    """The measurement aid behind the permutes' ceiling: a read-only kernel, so all there is to check is
    that it runs over the table it is given and that sizes it cannot take are refused before any launch."""
    rows, row_bytes = 4096, 1024
    table = torch.ones(rows * row_bytes // 4, dtype=torch.float32, device="cuda:0")
    order = torch.randperm(rows, device="cuda:0").to(torch.int32)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    for streaming in (0, 1):
        B.bigmac_gather_probe(table, order, rows, row_bytes, streaming, sink)
    torch.cuda.synchronize()
    assert int(sink.item()) == 0
    for bad_rows, bad_bytes in ((rows + 4, row_bytes), (rows, row_bytes + 16), (0, row_bytes), (rows, 0)):
        with pytest.raises(RuntimeError):
            B.bigmac_gather_probe(table, order, bad_rows, bad_bytes, 0, sink)


def test_run_to_run_determinism():
    wl = synth.small(T=700, d=256, r=128, N=16, k=4, h=256, zipf_s=1.2)
    data = synth.generate(wl)
    outs = []
    for _ in range(2):
        layer = DeviceLayer(wl, data)
        layer.forward(training=True)
        layer.alloc_grads()
        layer.backward()
        torch.cuda.synchronize()
        outs.append([layer.y.clone(), layer.dx.clone()] + [layer.grads[n].clone() for n in sorted(layer.grads)])
    for u, v in zip(*outs):
        assert torch.equal(u, v)


def test_identity_projections_reduce_to_fine_grained(oracle):
    # r = d and W_down = W_up = I: the BigMac layer is the fine-grained top-k MoE of its experts
    rng = np.random.default_rng(2)
    wl = synth.small(T=150, d=128, r=128, N=8, k=2, h=64)
    data = synth.generate(wl)
    data["w_down"] = np.eye(128, dtype=np.float32)
    data["w_up"] = np.eye(128, dtype=np.float32)
    y = host(DeviceLayer(wl, data).forward(training=False))
    fg = dict(data, cdac_w1=data["w1"], cdac_w2=data["w2"])
    wl_fg = synth.small(T=150, d=128, r=64, N=8, k=2, h=64)      # expert d=128 -> r=64 -> d
    y_fg = host(DeviceLayer(wl_fg, fg, order=B.ORDER_CDAC).forward(training=False))
    torch.cuda.synchronize()
    ref = oracle.cdac_forward(data["x"], data["w_gate"], None, data["w1"], data["w2"], 2)
    assert rel_err(y, ref) < TOL and rel_err(y_fg, ref) < TOL
    assert rel_err(y, y_fg) < TOL


@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_small_fine_grained_layer(oracle, dtype):
    print("small CDAC layer", dtype, flush=True)
    wl = synth.small(T=210, d=128, r=64, N=8, k=3, h=128, dtype=dtype)
    data = add_cdac_weights(synth.generate(wl))
    layer = DeviceLayer(wl, data, order=B.ORDER_CDAC)
    tol = TOL if dtype == B.BF16 else 1e-4
    y = host(layer.forward(training=True))
    torch.cuda.synchronize()
    ref = oracle.cdac_forward(data["x"], data["w_gate"], None, data["cdac_w1"], data["cdac_w2"], wl.k)
    assert rel_err(y, ref) < tol
    idx = check_routing(oracle, layer, data)
    g_ref = oracle.cdac_backward(data["x"], data["dy"], data["w_gate"], None, data["cdac_w1"], data["cdac_w2"], wl.k)
    layer.alloc_grads()
    layer.backward()
    torch.cuda.synchronize()
    assert rel_err(host(layer.dx), g_ref["dx"]) < tol
    grads = {n: host(layer.grads[n]) for n in ("d_w_gate", "d_w1", "d_w2")}
    counts = expert_effective_rows(oracle, data, wl)
    check_weight_grads(grads, g_ref, counts, tol, dcca=False, few_rows=dtype == B.BF16 and few_rows_per_expert(counts))


def test_tiny_fp32_workload_full(oracle):
    wl = synth.WORKLOADS["tiny_f32"]
    data = synth.generate(wl)
    layer = DeviceLayer(wl, data)
    y = host(layer.forward(training=True))
    torch.cuda.synchronize()
    assert rel_err(y, oracle_forward(oracle, data, wl.k)) < 1e-4
    check_routing(oracle, layer, data)
