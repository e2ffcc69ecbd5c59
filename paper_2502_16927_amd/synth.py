"""Seeded synthetic inputs for the BigMac layer (shapes of the paper's GPT-style MoE workloads).

This module only draws random tensors and rounds them once to the run's storage type.  It
holds none of the layer's arithmetic, so both the CPU oracle's tests and the HIP path's
tests/benchmark may draw their inputs from it.

Letters: T tokens, d model width, r low (dispatch) width, N experts, k experts per token,
h expert hidden width.  The paper's downscaling factor (Table 2, "r") is r/d here; every
workload keeps it at 0.25 as in the paper's analysis (Section 3.3, Table 4).
"""
from __future__ import annotations

import dataclasses
import numpy as np

F32 = 0
BF16 = 1


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    T: int
    d: int
    r: int
    N: int
    k: int
    h: int
    dtype: int            # F32 or BF16 storage of activations and GEMM weights
    x_std: float          # token distribution N(0, x_std^2)
    backward: bool
    zipf_s: float = 0.0   # >0: add a log-Zipf bias to the router logits
    index: int = 0        # seed offset

    def with_T(self, T: int) -> "Workload":
        return dataclasses.replace(self, T=T, name=f"{self.name}_T{T}")


# The five workloads the build is measured on.  Index = position in that list.
WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", T=256, d=256, r=64, N=8, k=2, h=256, dtype=F32,
                         x_std=0.02, backward=False, index=0),
    "gpt_medium": Workload("gpt_medium", T=8192, d=1024, r=256, N=64, k=8, h=1024, dtype=BF16,
                           x_std=1.0, backward=True, index=1),
    "gpt_xl": Workload("gpt_xl", T=16384, d=2048, r=512, N=64, k=6, h=2048, dtype=BF16,
                       x_std=1.0, backward=True, index=2),
    "decode": Workload("decode", T=2048, d=4096, r=1024, N=64, k=8, h=4096, dtype=BF16,
                       x_std=1.0, backward=False, index=3),
    "zipf_stress": Workload("zipf_stress", T=32768, d=4096, r=1024, N=128, k=8, h=2048,
                            dtype=BF16, x_std=1.0, backward=True, zipf_s=1.2, index=4),
}
# A further structure built from the same kernels: the vanilla MoE layer (Fig. 2a: few experts,
# each a full-width d -> 4d -> d FFN, top-2, no shared projections).  It runs in the CDAC order
# with the expert hidden width in `r` (and h = d, so that the expert matrices can be drawn as
# the swapped BigMac ones).
NEXT_WORKLOADS = {
    "vanilla_moe": Workload("vanilla_moe", T=8192, d=1024, r=4096, N=8, k=2, h=1024, dtype=BF16,
                            x_std=1.0, backward=True, index=5),
    # The two larger base models of the paper's training comparison (Fig. 3: GPT3-2.7B and
    # GPT3-6.7B widths), as BigMac layers with the same expert count, top-8 and r/d = 1/4.
    "gpt_2p7b": Workload("gpt_2p7b", T=8192, d=2560, r=640, N=64, k=8, h=2560, dtype=BF16,
                         x_std=1.0, backward=True, index=6),
    "gpt_6p7b": Workload("gpt_6p7b", T=8192, d=4096, r=1024, N=64, k=8, h=4096, dtype=BF16,
                         x_std=1.0, backward=True, index=7),
}
DECODE_T_SWEEP = (32, 128, 512, 2048)
W_STD = 0.02
BASE_SEED = 1234  # the seed the paper's pre-training setup lists (Table 5)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays in an fp32 array."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    out = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return out.view(np.float32)


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Upper 16 bits of already bf16-representable fp32 values, as uint16 (device storage)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(rng: np.random.Generator, shape, std: float, chunk_rows: int = 1 << 14) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(shape[0], -1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        flat[r0:r1] = rng.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32) * np.float32(std)
    return out


def generate(wl: Workload, seed: int | None = None, with_dy: bool | None = None) -> dict:
    """Draw all tensors of one layer call as fp32 numpy arrays already rounded to wl.dtype.

    One generator stream per tensor (spawned from one seed) so that changing a shape does not
    shift the other tensors.  w_gate and gate_bias always stay fp32.
    """
    seed = BASE_SEED + wl.index if seed is None else seed
    streams = np.random.SeedSequence(seed).spawn(9)
    g = [np.random.default_rng(s) for s in streams]
    rnd = round_to_bf16 if wl.dtype == BF16 else (lambda a: a)
    out = {
        "x": rnd(_normal(g[0], (wl.T, wl.d), wl.x_std)),
        "w_gate": _normal(g[1], (wl.d, wl.N), W_STD),
        "w_down": rnd(_normal(g[2], (wl.d, wl.r), W_STD)),
        "w_up": rnd(_normal(g[3], (wl.r, wl.d), W_STD)),
        "w1": rnd(_normal(g[4], (wl.N, wl.r, wl.h), W_STD)),
        "w2": rnd(_normal(g[5], (wl.N, wl.h, wl.r), W_STD)),
        "gate_bias": None,
    }
    if wl.zipf_s > 0.0:
        rank = g[6].permutation(wl.N).astype(np.float64)
        out["gate_bias"] = (-wl.zipf_s * np.log1p(rank)).astype(np.float32)
    if wl.backward if with_dy is None else with_dy:
        out["dy"] = rnd(_normal(g[7], (wl.T, wl.d), 1.0))
    return out


def small(T=96, d=128, r=64, N=8, k=2, h=128, dtype=BF16, x_std=1.0, zipf_s=0.0, index=100) -> Workload:
    """A workload small enough for the oracle to finish in well under a second."""
    return Workload(f"small_T{T}_d{d}_r{r}_N{N}_k{k}_h{h}", T, d, r, N, k, h, dtype, x_std, True,
                    zipf_s, index)
