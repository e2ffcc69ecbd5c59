"""The allocation-free dispatch (bigmac_dispatch_static) against bigmac_dispatch: same permutation
and rows, bit for bit, on two calls in a row of which the second is smaller (the library's static
scratch keeps the first call's contents), also in capacity mode, and the size limit's error."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2502_16927_amd import binding as B
from paper_2502_16927_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_both(T, k, N, width, dtype, seed, capacity=0):
    rng = np.random.default_rng(seed)
    skew = rng.random(N) ** 3 + 1e-3
    idx_np = np.stack([rng.choice(N, size=k, replace=False, p=skew / skew.sum()) for _ in range(T)]).astype(np.int32)
    xl_np = rng.standard_normal((T, width)).astype(np.float32)
    if dtype == B.BF16:
        xl_np = synth.round_to_bf16(xl_np)
    dims = B.make_dims(T, 64, width, N, k, 64, dtype, capacity=capacity)
    idx = torch.from_numpy(idx_np).to(DEV)
    xl = B.to_device(xl_np, dtype)
    outs = []
    for static in (False, True):
        xp = torch.zeros((T * k, width), dtype=B.act_dtype(dtype), device=DEV)
        off = torch.zeros(N + 1, dtype=torch.int32, device=DEV)
        slot = torch.zeros((T, k), dtype=torch.int32, device=DEV)
        src = torch.full((T * k,), -7, dtype=torch.int32, device=DEV)
        if static:
            B.bigmac_dispatch_static(dims, xl, idx, xp, off, slot, src)
        else:
            ws = B.alloc_bytes(B.workspace_bytes(dims, B.WS_DISPATCH))
            B.bigmac_dispatch(dims, xl, idx, xp, off, slot, src, ws)
        torch.cuda.synchronize()
        outs.append((off, slot, src, xp))
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    return outs[1]


@pytest.mark.parametrize("dtype", [B.BF16, B.F32])
def test_static_dispatch_matches_dispatch_twice_in_a_row(oracle, dtype):
    print(f"allocation-free dispatch, dtype {dtype}: 12000 pairs then 6000 pairs", flush=True)
    # both sizes take the three-kernel counting sort, whose counters live in the scratch
    off, slot, src, xp = run_both(3000, 4, 16, 192, dtype, seed=1)
    assert int(off[-1]) == 12000
    off, slot, src, xp = run_both(1500, 4, 16, 192, dtype, seed=2)
    assert int(off[-1]) == 6000
    print("capacity mode, then the one-workgroup sort of a decode batch", flush=True)
    off, _, _, _ = run_both(2500, 4, 16, 64, dtype, seed=3, capacity=300)
    assert 0 < int(off[-1]) < 10000
    run_both(100, 4, 16, 64, dtype, seed=4)


def test_static_dispatch_rejects_what_does_not_fit():
    L = B.lib()
    fake = ctypes.c_void_p(4096)             # never dereferenced: the size is checked first
    big = B.make_dims(1 << 22, 64, 64, 1024, 8, 64)      # 2^25 pairs / 1024 x 1024 experts x 4 bytes = 128 MiB of counters
    assert L.bigmac_dispatch_static(ctypes.byref(big), fake, fake, fake, fake, fake, fake, None) == -5
    assert "static scratch" in B.status_string(-5)
    ok = B.make_dims(128, 64, 64, 8, 2, 64)
    assert L.bigmac_dispatch_static(ctypes.byref(ok), fake, None, fake, fake, fake, fake, None) == -1
