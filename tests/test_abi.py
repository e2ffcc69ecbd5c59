"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
that include/bigmac.h declares, sizes and closed forms are sane, and bad arguments are turned
into error codes before anything is launched."""
import ctypes
import os
import re

import pytest

from paper_2502_16927_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "bigmac.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bigmac_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    L = B.lib()
    names = declared_functions()
    assert len(names) >= 11
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names
    assert B.STAGE_COUNT == len([1 for s in range(64) if B.stage_name(s) != "?"])


def test_status_strings_and_sizes():
    assert B.status_string(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert B.status_string(code) not in ("ok", "unknown status")
    d = B.make_dims(8192, 1024, 256, 64, 8, 1024)
    sizes = [B.workspace_bytes(d, k) for k in range(6)]
    assert all(s > 0 and s % 256 == 0 for s in sizes)
    Tk = 8192 * 8
    assert sizes[B.WS_ROUTE] == 8192 * 64 * 4
    # saved block holds x_perm, act, hact, o_perm (bf16) and the routing arrays
    assert sizes[B.WS_SAVED] >= 2 * Tk * (2 * 256 + 2 * 1024)
    lay = B.saved_layout(d)
    assert lay["topk_idx"] == 0 and lay["topk_w"] >= Tk * 4 and lay["slot_of"] > lay["expert_offsets"]


def test_closed_forms_of_table_3():
    # matrix FLOPs of a forward pass = (paper's 12 d^2 rho (k+1) per token for fwd+bwd) / 3
    d = B.make_dims(4096, 2048, 512, 64, 8, 2048)
    assert B.forward_matrix_flops(d) == 4096 * 12 * 2048 ** 2 * 0.25 * 9 / 3
    fine = B.make_dims(4096, 2048, 512, 64, 8, 2048, order=B.ORDER_CDAC)
    assert B.forward_matrix_flops(fine) == 4096 * 12 * 2048 ** 2 * 0.25 * 8 / 3
    # the four permutes move 8 * tokens * k * width bytes in bf16; BigMac moves r/d of the fine-grained layer
    assert B.permute_bytes(fine) == 8 * 4096 * 8 * 2048
    assert B.permute_bytes(d) / B.permute_bytes(fine) == 0.25


BAD_DIMS = [
    dict(T=0), dict(d=100), dict(r=32), dict(h=65), dict(k=0), dict(k=9, N=8), dict(N=2048), dict(k=65, N=128),
    dict(dtype=7), dict(act=3), dict(order=2), dict(flags=128), dict(T=1 << 29, k=8),
]


@pytest.mark.parametrize("bad", BAD_DIMS, ids=lambda b: "_".join(f"{k}{v}" for k, v in b.items()))
def test_bad_dims_are_rejected_before_any_launch(bad):
    base = dict(T=128, d=128, r=64, N=8, k=2, h=128, dtype=B.BF16, order=B.ORDER_DCCA, flags=0, act=0)
    base.update(bad)
    d = B.make_dims(**base)
    assert B.workspace_bytes(d, B.WS_LAYER_TRAIN) == 0
    L = B.lib()
    fake = ctypes.c_void_p(4096)             # never dereferenced: the dims are checked first
    rc = L.bigmac_route(ctypes.byref(d), fake, fake, None, fake, fake, None, fake, 1 << 30, None)
    assert rc in (-1, -3)
    rc = L.bigmac_combine(ctypes.byref(d), fake, fake, None, fake, None)
    assert rc in (-1, -3)


def test_null_pointers_and_small_workspaces_are_rejected():
    L = B.lib()
    d = B.make_dims(128, 128, 64, 8, 2, 128)
    fake = ctypes.c_void_p(4096)
    dp = ctypes.byref(d)
    assert L.bigmac_route(dp, None, fake, None, fake, fake, None, fake, 1 << 30, None) == -1
    assert L.bigmac_route(dp, fake, fake, None, fake, fake, None, None, 0, None) == -1      # no logits buffer, no workspace
    assert L.bigmac_route(dp, fake, fake, None, fake, fake, None, fake, 16, None) == -2
    assert L.bigmac_dispatch(dp, fake, None, fake, fake, fake, fake, fake, 1 << 30, None) == -1
    assert L.bigmac_dispatch(dp, fake, fake, None, fake, fake, fake, fake, 1 << 30, None) == -1  # x_low without x_perm
    assert L.bigmac_dispatch(dp, fake, fake, fake, fake, fake, fake, fake, 8, None) == -2
    assert L.bigmac_grouped_ffn(dp, fake, fake, fake, None, None, None, None, fake, fake, 1 << 30, None) == -1
    assert L.bigmac_grouped_ffn(dp, fake, fake, fake, fake, None, None, None, fake, fake, 64, None) == -2
    assert L.bigmac_combine(dp, None, fake, None, fake, None) == -1
    p = B.Params(None, None, None, None, None, None, None, None)
    assert L.bigmac_layer_forward(dp, ctypes.byref(p), fake, fake, None, fake, 1 << 40, None) == -1
    p = B.Params(4096, 4096, 4096, None, 4096, 4096, None, None)
    assert L.bigmac_layer_forward(dp, ctypes.byref(p), fake, fake, None, fake, 1024, None) == -2
    assert L.bigmac_layer_backward(dp, ctypes.byref(p), fake, fake, None, fake, fake, fake, fake, fake, fake, None, None, fake, 1 << 40, None) == -1
    assert L.bigmac_layer_backward(dp, ctypes.byref(p), fake, fake, fake, fake, fake, fake, fake, fake, fake, None, None, fake, 1024, None) == -2
    odd = B.make_dims(128, 128, 64, 12, 2, 128)                                             # N not a multiple of 8
    assert L.bigmac_layer_backward(ctypes.byref(odd), ctypes.byref(p), fake, fake, fake, fake, fake, fake, fake, fake, fake, None, None, fake, 1 << 40, None) == -3
    fg = B.make_dims(128, 128, 64, 8, 2, 128, order=B.ORDER_CDAC, flags=B.FLAG_OUT_BF16)
    assert B.workspace_bytes(fg, B.WS_LAYER_FORWARD) == 0


def test_where_the_dispatch_step_runs():
    """bigmac_dispatch_folding: host logic only.  Forward-only bf16 calls fold the dispatch into the
    expert-up product; DCCA training calls into the descending projection unless the router reads
    x', the flag forbids it, the storage is fp32 or the projection is summed from K slices."""
    big = dict(T=32768, d=4096, r=1024, N=128, k=8, h=2048)
    assert B.dispatch_folding(B.make_dims(**big), training=True) == 2
    assert B.dispatch_folding(B.make_dims(**big), training=False) == 1
    assert B.dispatch_folding(B.make_dims(**big, flags=B.FLAG_NO_FUSED_DISPATCH), training=True) == 0
    assert B.dispatch_folding(B.make_dims(**big, flags=B.FLAG_NO_FUSED_DISPATCH), training=False) == 0
    assert B.dispatch_folding(B.make_dims(**big, flags=B.FLAG_ROUTE_LOW), training=True) == 0
    assert B.dispatch_folding(B.make_dims(4096, 4096, 4096, 8, 2, 4096, order=B.ORDER_CDAC), training=True) == 0
    assert B.dispatch_folding(B.make_dims(256, 256, 64, 8, 2, 256, dtype=B.F32), training=True) == 0
    assert B.dispatch_folding(B.make_dims(256, 256, 64, 8, 2, 256, dtype=B.F32), training=False) == 0
    assert B.dispatch_folding(B.make_dims(8192, 1024, 256, 64, 8, 1024), training=True) == 2
    assert B.dispatch_folding(B.make_dims(200, 768, 256, 8, 2, 128), training=True) == 0         # the projection is summed from K slices
    assert B.dispatch_folding(B.make_dims(262144, 4096, 1024, 128, 8, 2048), training=True) == 0  # permuted copy of 4 GiB: past one 32-bit offset
    assert B.dispatch_folding(B.make_dims(262144, 4096, 1024, 128, 8, 2048), training=False) == 1  # x' is 512 MiB
    assert B.dispatch_folding(B.make_dims(262144, 4096, 4096, 128, 8, 4096, order=B.ORDER_CDAC), training=False) == 0   # x is 2 GiB
