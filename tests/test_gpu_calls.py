"""Parity of each C-ABI call against the CPU oracle on small seeded inputs that still span
several tiles and ragged tails.  Integer results bit-exact; floating point within 2e-2 of the
oracle tensor's RMS (max-abs)."""
import numpy as np
import pytest
import torch

from paper_2502_16927_amd import binding as B
from paper_2502_16927_amd import synth
from gpu_util import TOL, host, rel_err

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

ROUTE_CASES = [
    # T, d, N, k, dtype, zipf
    (1, 64, 8, 2, B.BF16, 0.0),
    (37, 128, 8, 8, B.F32, 0.0),
    (300, 256, 64, 8, B.BF16, 0.0),
    (257, 192, 24, 5, B.BF16, 1.2),
    (130, 512, 128, 8, B.BF16, 1.2),
    (70, 64, 200, 64, B.F32, 0.0),
    (33, 1024, 1024, 3, B.BF16, 0.0),
]


@pytest.mark.parametrize("T,d,N,k,dtype,zipf", ROUTE_CASES)
def test_route_matches_oracle(oracle, T, d, N, k, dtype, zipf):
    print(f"route T={T} d={d} N={N} k={k} dtype={dtype}", flush=True)
    wl = synth.small(T=T, d=d, r=64, N=N, k=k, h=64, dtype=dtype, zipf_s=zipf)
    data = synth.generate(wl)
    dims = B.dims_of(wl)
    x = B.to_device(data["x"], dtype)
    wg = B.to_device(data["w_gate"], B.F32)
    bias = B.to_device(data["gate_bias"], B.F32)
    idx = torch.empty((T, k), dtype=torch.int32, device=DEV)
    w = torch.empty((T, k), dtype=torch.float32, device=DEV)
    logits = torch.empty((T, N), dtype=torch.float32, device=DEV)
    B.bigmac_route(dims, x, wg, bias, idx, w, logits)
    torch.cuda.synchronize()
    ref_idx, ref_gate, ref_logits = oracle.route(data["x"], data["w_gate"], data["gate_bias"], k)
    assert np.array_equal(host(logits).view(np.uint32), ref_logits.view(np.uint32)), "logits differ in some bit"
    assert np.array_equal(host(idx), ref_idx)
    assert np.abs(host(w) - ref_gate).max() < 1e-6
    # without a logits buffer the call uses its workspace
    idx2 = torch.empty_like(idx)
    w2 = torch.empty_like(w)
    ws = B.alloc_bytes(B.workspace_bytes(dims, B.WS_ROUTE))
    B.bigmac_route(dims, x, wg, bias, idx2, w2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(w, w2)


def test_route_ties_and_order_cases(oracle):
    # duplicated router columns give exactly equal logits: the lowest index must win
    rng = np.random.default_rng(3)
    T, d = 96, 128
    x = synth.round_to_bf16(rng.standard_normal((T, d)).astype(np.float32))
    col = rng.standard_normal((d, 3)).astype(np.float32)
    wg = np.ascontiguousarray(np.stack([col[:, 0], col[:, 1], col[:, 2], col[:, 2], col[:, 1], col[:, 0], col[:, 1], col[:, 0]], axis=1))
    dims = B.make_dims(T, d, 64, 8, 4, 64, B.BF16)
    idx = torch.empty((T, 4), dtype=torch.int32, device=DEV)
    w = torch.empty((T, 4), dtype=torch.float32, device=DEV)
    lg = torch.empty((T, 8), dtype=torch.float32, device=DEV)
    B.bigmac_route(dims, B.to_device(x, B.BF16), B.to_device(wg, B.F32), None, idx, w, lg)
    torch.cuda.synchronize()
    ref_idx, ref_gate, ref_logits = oracle.route(x, wg, None, 4)
    assert np.array_equal(host(lg).view(np.uint32), ref_logits.view(np.uint32))
    assert np.array_equal(host(idx), ref_idx)
    # the same across the two registers of the 65..128-expert path: every logit has equal copies in
    # both halves, more picks than distinct values, and the full k = 64 of 128
    for N, k in ((100, 33), (128, 64), (65, 2)):
        col = rng.standard_normal((d, 7)).astype(np.float32)
        wg = np.ascontiguousarray(col[:, np.arange(N) % 7])
        dims = B.make_dims(T, d, 64, N, k, 64, B.BF16)
        idx = torch.empty((T, k), dtype=torch.int32, device=DEV)
        w = torch.empty((T, k), dtype=torch.float32, device=DEV)
        lg = torch.empty((T, N), dtype=torch.float32, device=DEV)
        B.bigmac_route(dims, B.to_device(x, B.BF16), B.to_device(wg, B.F32), None, idx, w, lg)
        torch.cuda.synchronize()
        ref_idx, ref_gate, _ = oracle.route(x, wg, None, k)
        assert np.array_equal(host(idx), ref_idx), (N, k)
        assert np.abs(host(w) - ref_gate).max() < 1e-6
    # absorption cases where the summation order shows
    xo = np.zeros((3, d), np.float32)
    xo[0, 0], xo[0, 1], xo[0, 64] = 1e8, 1.0, -1e8
    xo[1, 0], xo[1, 1], xo[1, 32] = 1e8, 1.0, -1e8
    xo[2, 0], xo[2, 8], xo[2, 16] = 1e8, 1.0, -1e8
    ones = np.ones((d, 8), np.float32)
    dims = B.make_dims(3, d, 64, 8, 1, 64, B.F32)
    lg = torch.empty((3, 8), dtype=torch.float32, device=DEV)
    B.bigmac_route(dims, B.to_device(xo, B.F32), B.to_device(ones, B.F32), None,
                   torch.empty((3, 1), dtype=torch.int32, device=DEV), torch.empty((3, 1), dtype=torch.float32, device=DEV), lg)
    torch.cuda.synchronize()
    assert np.array_equal(host(lg), oracle.router_logits(xo, ones)) and np.all(host(lg) == 1.0)


PERM_CASES = [(1, 1, 1), (5, 2, 3), (700, 8, 64), (1025, 6, 24), (4096, 8, 128), (3000, 2, 1000), (513, 64, 64),
              # up to 4096 pairs one workgroup does the whole sort: 1, 2 and 4 rounds of 1024 pairs, a full last
              # round, 3 rounds needed, the counter limit (512 x 8 pairs, 128 experts) and just past it
              (128, 8, 64), (130, 8, 64), (512, 8, 64), (300, 8, 100), (512, 8, 128), (512, 8, 129), (37, 3, 500)]


@pytest.mark.parametrize("T,k,N", PERM_CASES)
@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_dispatch_permutation_and_rows(oracle, T, k, N, dtype):
    print(f"dispatch T={T} k={k} N={N} dtype={dtype}", flush=True)
    rng = np.random.default_rng(T * 31 + k)
    skew = rng.random(N) ** 3 + 1e-3                       # uneven expert popularity, some nearly empty
    idx_np = np.stack([rng.choice(N, size=k, replace=False, p=skew / skew.sum()) for _ in range(T)]).astype(np.int32)
    width = 192
    dims = B.make_dims(T, 64, width, N, k, 64, dtype)
    xl_np = rng.standard_normal((T, width)).astype(np.float32)
    if dtype == B.BF16:
        xl_np = synth.round_to_bf16(xl_np)
    idx = torch.from_numpy(idx_np).to(DEV)
    xl = B.to_device(xl_np, dtype)
    xp = torch.empty((T * k, width), dtype=B.act_dtype(dtype), device=DEV)
    off = torch.empty(N + 1, dtype=torch.int32, device=DEV)
    slot = torch.empty((T, k), dtype=torch.int32, device=DEV)
    src = torch.empty(T * k, dtype=torch.int32, device=DEV)
    ws = B.alloc_bytes(B.workspace_bytes(dims, B.WS_DISPATCH))
    B.bigmac_dispatch(dims, xl, idx, xp, off, slot, src, ws)
    torch.cuda.synchronize()
    r_off, r_slot, r_src = oracle.permutation(idx_np, N)
    assert np.array_equal(host(off), r_off)
    assert np.array_equal(host(slot), r_slot)
    assert np.array_equal(host(src), r_src)
    assert np.array_equal(host(xp), oracle.dispatch(xl_np, r_slot))
    # permutation only
    slot2 = torch.empty_like(slot)
    B.bigmac_dispatch(dims, None, idx, None, off, slot2, src, ws)
    torch.cuda.synchronize()
    assert torch.equal(slot, slot2)
    # round trip: unit-weight combine of the dispatched rows gives k * x_low
    y = torch.empty((T, width), dtype=torch.float32, device=DEV)
    B.bigmac_combine(dims, xp, slot, None, y)
    torch.cuda.synchronize()
    assert np.abs(host(y) - k * xl_np.astype(np.float64)).max() <= 1e-5 * k * np.abs(xl_np).max()


@pytest.mark.parametrize("T,k,N,width", [(50, 2, 8, 64), (333, 8, 64, 256), (129, 6, 16, 1024)])
@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_combine_matches_oracle(oracle, T, k, N, width, dtype):
    print(f"combine T={T} k={k} width={width} dtype={dtype}", flush=True)
    rng = np.random.default_rng(width + T)
    idx_np = np.stack([rng.permutation(N)[:k] for _ in range(T)]).astype(np.int32)
    _, slot_np, _ = oracle.permutation(idx_np, N)
    o_np = rng.standard_normal((T * k, width)).astype(np.float32)
    if dtype == B.BF16:
        o_np = synth.round_to_bf16(o_np)
    g = rng.random((T, k)).astype(np.float32)
    g /= g.sum(1, keepdims=True)
    dims = B.make_dims(T, 64, width, N, k, 64, dtype)
    y = torch.empty((T, width), dtype=torch.float32, device=DEV)
    B.bigmac_combine(dims, B.to_device(o_np, dtype), torch.from_numpy(slot_np).to(DEV), torch.from_numpy(g).to(DEV), y)
    torch.cuda.synchronize()
    ref = oracle.combine(o_np.astype(np.float64), slot_np, g.astype(np.float64))
    assert rel_err(host(y), ref) < 1e-5


FFN_CASES = [
    # T, r(win), h(hid), N, k, dtype, order
    (64, 64, 64, 4, 2, B.BF16, B.ORDER_DCCA),
    (300, 128, 320, 8, 3, B.BF16, B.ORDER_DCCA),
    (500, 256, 192, 24, 8, B.BF16, B.ORDER_DCCA),
    (200, 64, 128, 8, 2, B.F32, B.ORDER_DCCA),
    (260, 64, 64, 8, 4, B.BF16, B.ORDER_CDAC),      # expert d=256 -> r=64 -> d
    # enough rows, tiles and K for the 256-row workgroup tiles: first product tall, second not ...
    (2560, 512, 2048, 16, 8, B.BF16, B.ORDER_DCCA),
    # ... and the other way round
    (5120, 1024, 512, 32, 8, B.BF16, B.ORDER_DCCA),
]


@pytest.mark.parametrize("T,r,h,N,k,dtype,order", FFN_CASES)
def test_grouped_ffn_matches_oracle(oracle, T, r, h, N, k, dtype, order):
    print(f"grouped_ffn T={T} r={r} h={h} N={N} k={k} dtype={dtype} order={order}", flush=True)
    rng = np.random.default_rng(T + r)
    d = 256
    win, hid = (r, h) if order == B.ORDER_DCCA else (d, r)
    rnd = synth.round_to_bf16 if dtype == B.BF16 else (lambda a: a)
    skew = rng.random(N) ** 2 + 1e-3
    if N >= 4:
        skew[1] = 0.0                                       # an expert with no rows at all
    idx_np = np.stack([rng.choice(N, size=k, replace=False, p=skew / skew.sum()) for _ in range(T)]).astype(np.int32)
    off_np, slot_np, _ = oracle.permutation(idx_np, N)
    xp_np = rnd(rng.standard_normal((T * k, win)).astype(np.float32))
    w1_np = rnd((rng.standard_normal((N, win, hid)) * 0.1).astype(np.float32))
    w2_np = rnd((rng.standard_normal((N, hid, win)) * 0.1).astype(np.float32))
    dims = B.make_dims(T, d, r, N, k, h, dtype, order)
    o = torch.empty((T * k, win), dtype=B.act_dtype(dtype), device=DEV)
    a = torch.empty((T * k, hid), dtype=B.act_dtype(dtype), device=DEV)
    ws = B.alloc_bytes(B.workspace_bytes(dims, B.WS_GROUPED_FFN))
    args = (B.to_device(xp_np, dtype), torch.from_numpy(off_np).to(DEV), B.to_device(w1_np, dtype), B.to_device(w2_np, dtype))
    B.bigmac_grouped_ffn(dims, *args, a, o, ws)
    torch.cuda.synchronize()
    ref_o, ref_a = oracle.expert_rows(xp_np, off_np, w1_np, w2_np, want_a=True)
    tol = TOL if dtype == B.BF16 else 1e-4
    assert rel_err(host(a), ref_a) < tol
    assert rel_err(host(o), ref_o) < tol
    o2 = torch.empty_like(o)
    B.bigmac_grouped_ffn(dims, *args, None, o2, ws)        # inference: no pre-activation kept
    torch.cuda.synchronize()
    assert torch.equal(o, o2)


def test_mfma_probe_counts_its_flops():
    sink = torch.zeros(1, dtype=torch.float32, device=DEV)
    flops = B.bigmac_mfma_probe(8, 10, sink)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 10 * 16 * 2.0 * 32 * 32 * 16
    assert float(sink.item()) == 0.0            # never written
    with pytest.raises(B.BigmacError):
        B.bigmac_mfma_probe(0, 10, sink)
    with pytest.raises(B.BigmacError):
        B.bigmac_mfma_probe(8, 0, sink)
