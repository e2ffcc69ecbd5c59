#!/usr/bin/env python3
"""Benchmark of the BigMac MoE layer on one MI355X: tokens/s of one layer step (forward +
backward on workloads that train, forward only otherwise) on seeded synthetic inputs resident in
HBM, the roofline of the kernel that dominates the step, and the CPU oracle timed beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload zipf_stress] [--order dcca|cdac]

Prints ONE JSON line.  Runs on one GPU only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM = 8.0e12          # bytes/s, MI355X HBM3E
PEAK_MFMA_BF16 = 2.5e15    # flop/s, dense bf16 MFMA
PEAK_ALU_F32 = 157.3e12    # flop/s, published fp32 vector peak (unpacked v_fmac_f32 measured at 146 TFLOP/s with two waves per SIMD)


# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE x 2.0 KiB + WRITE_SIZE x 1.0 KiB, the
# factors a plain 512 MiB copy gives: `bench.py --calibrate-copy`), for the kernels that can
# dominate a workload.  A counter run cannot be part of a timed run; these are the figures of
# the committed summaries of those runs (the *_hbm_traffic files under profiles/).
MEASURED_TRAFFIC = {   # stage -> (MiB read, MiB written) per launch
    ("gpt_medium", "dcca"): {"source": "profiles/gpt_medium_hbm_traffic.md",
                             "expert_up": (98.9, 256.2), "expert_down": (168.5, 64.1), "bwd_down_dgrad": (195.9, 128.2),
                             "bwd_down_wgrad": (160.8, 64.0), "bwd_up_wgrad": (160.3, 64.0), "bwd_up_dgrad": (170.7, 64.1)},
    ("zipf_stress", "dcca"): {"source": "profiles/zipf_stress_hbm_traffic.md",
                              "expert_up": (3834.0, 2048.5), "expert_down": (2061.0, 1024.2), "bwd_down_dgrad": (3480.6, 1161.2),
                              "bwd_down_wgrad": (2446.9, 1024.0), "bwd_up_wgrad": (3409.1, 1024.1), "bwd_up_dgrad": (2066.0, 1024.2)},
    ("gpt_xl", "dcca"): {"source": "profiles/gpt_xl_hbm_traffic.md",
                         "expert_up": (252.3, 768.3), "expert_down": (581.7, 192.1), "bwd_down_dgrad": (633.4, 384.2),
                         "bwd_down_wgrad": (570.9, 256.0), "bwd_up_wgrad": (481.7, 256.0), "bwd_up_dgrad": (581.6, 192.1)},
}


def stage_work(wl, order_cdac: bool, training: bool, wire_bf16: bool = False):
    """Algorithmic work per stage: (kind, flops, bytes).  Bytes are compulsory traffic: every
    input read once, every output written once, real rows only.  e = bytes per stored element,
    ew = bytes per element of the rows that return through the second All-to-All (expert outputs)
    and of their backward counterpart (fp32 unless the all-bf16 wire format is asked for)."""
    T, d, r, N, k, h = wl.T, wl.d, wl.r, wl.N, wl.k, wl.h
    e = 2 if wl.dtype == 1 else 4
    ew = 2 if (e == 2 and wire_bf16) else 4
    Tk = T * k
    win, hid = (d, r) if order_cdac else (r, h)
    low = 2 * r if e == 2 else r          # y' and dx' travel as (hi | lo) bf16 pairs
    W = {}
    W["router_logits"] = ("alu", 2.0 * T * d * N, T * d * e + d * N * 4 + T * N * 4)
    W["topk_gate"] = ("hbm", 0.0, T * N * 4 + 8 * Tk)
    W["descend"] = ("mfma", 2.0 * T * d * r, T * d * e + d * r * e + T * r * e)
    W["permutation"] = ("hbm", 0.0, 4 * Tk * 4)
    W["dispatch"] = ("hbm", 0.0, (T + Tk) * win * e + 4 * Tk)
    W["expert_up"] = ("mfma", 2.0 * Tk * win * hid, Tk * win * e + N * win * hid * e + Tk * hid * e * (2 if training else 1))
    W["expert_down"] = ("mfma", 2.0 * Tk * hid * win, Tk * hid * e + N * win * hid * e + Tk * win * ew)
    W["combine"] = ("hbm", 2.0 * Tk * win, Tk * win * ew + T * (low * e if not order_cdac else d * 4) + 8 * Tk)
    W["ascend"] = ("mfma", 2.0 * T * r * d, T * low * e + r * d * e + T * d * 4)
    W["bwd_ascend_dgrad"] = ("mfma", 2.0 * T * d * r, T * d * e + r * d * e + T * r * 4)
    W["bwd_ascend_wgrad"] = ("mfma", 2.0 * T * r * d, T * r * e + T * d * e + r * d * 4)
    W["bwd_combine"] = ("hbm", 4.0 * Tk * win, T * win * 4 + Tk * win * ew + Tk * win * e + 12 * Tk)
    W["bwd_down_dgrad"] = ("mfma", 2.0 * Tk * win * hid, Tk * win * e + N * win * hid * e + 2 * Tk * hid * e)
    W["bwd_down_wgrad"] = ("mfma", 2.0 * Tk * win * hid, Tk * hid * e + Tk * win * e + N * win * hid * 4)
    W["bwd_up_wgrad"] = ("mfma", 2.0 * Tk * win * hid, Tk * hid * e + Tk * win * e + N * win * hid * 4)
    W["bwd_up_dgrad"] = ("mfma", 2.0 * Tk * win * hid, Tk * hid * e + N * win * hid * e + Tk * win * ew)
    W["bwd_dispatch"] = ("hbm", 1.0 * Tk * win, Tk * win * ew + T * (low * e if not order_cdac else d * 4) + 4 * Tk)
    W["bwd_gate"] = ("hbm", 2.0 * Tk * d, T * d * 4 + T * N * e + 12 * Tk)
    W["bwd_router_wgrad"] = ("mfma", 2.0 * T * d * N, T * d * e + T * N * e + d * N * 4)
    W["bwd_descend_wgrad"] = ("mfma", 2.0 * T * d * r, T * d * e + T * r * e + d * r * 4)
    W["bwd_descend_dgrad"] = ("mfma", 2.0 * T * r * d, T * low * e + d * r * e + 2 * T * d * 4)
    W["bwd_output_cast"] = ("hbm", 0.0, 3 * T * d * 4)
    return W


def roofline_of(name, kind, flops, nbytes, seconds):
    """The roofline that bounds this kernel: whichever of its algorithmic flops or bytes takes
    longer at the chip's peak."""
    peak_f = PEAK_ALU_F32 if kind == "alu" else PEAK_MFMA_BF16
    t_f = flops / peak_f if flops else 0.0
    t_b = nbytes / PEAK_HBM
    if kind != "hbm" and t_f >= t_b:
        achieved, peak = flops / seconds / 1e12, peak_f / 1e12
        return {"kernel": name, "bound": "alu" if kind == "alu" else "mfma", "achieved": achieved, "peak": peak,
                "unit": "TFLOP/s", "frac": achieved / peak, "traffic": None, "algorithmic_flops": flops,
                "algorithmic_bytes": nbytes, "avg_ms": seconds * 1e3}
    achieved, peak = nbytes / seconds / 1e9, PEAK_HBM / 1e9
    return {"kernel": name, "bound": "hbm", "achieved": achieved, "peak": peak, "unit": "GB/s", "frac": achieved / peak,
            "traffic": None, "algorithmic_flops": flops, "algorithmic_bytes": nbytes, "avg_ms": seconds * 1e3}


def cpu_baseline(wl, data, sample_tokens: int, training: bool):
    """The oracle as it stands, timed on the host cores on a bounded token sample."""
    import numpy as np
    from oracle import cpu_oracle
    n = min(sample_tokens, wl.T)
    sel = np.linspace(0, wl.T - 1, n).astype(np.int32)
    t0 = time.perf_counter()
    cpu_oracle.bigmac_forward(data["x"], data["w_gate"], data["gate_bias"], data["w_down"], data["w_up"],
                              data["w1"], data["w2"], wl.k, sel=sel)
    if training:
        cpu_oracle.bigmac_backward(data["x"], data["dy"], data["w_gate"], data["gate_bias"], data["w_down"],
                                   data["w_up"], data["w1"], data["w2"], wl.k, sel=sel)
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "tokens/s", "cores": cpu_oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} evenly spaced tokens of the same workload, forward{'+backward' if training else ''}, "
                      f"{dt:.1f} s wall"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="zipf_stress",
                    help="zipf_stress (default: the largest of the five workloads), gpt_xl, gpt_medium, decode, tiny_f32, "
                         "or one of gpt_2p7b, gpt_6p7b, vanilla_moe")
    ap.add_argument("--blocks", type=int, default=3,
                    help="timed blocks of --steps graph replays each: the first is the reported value, all of them "
                         "are listed with their median and minimum")
    ap.add_argument("--wire-bf16", action="store_true",
                    help="all-bf16 wire format (BIGMAC_FLAG_WIRE_BF16): expert outputs and the gradient of the dispatched "
                         "rows in bf16 instead of fp32; less permute traffic, y and dx no longer within 2e-2 at the widest shapes")
    ap.add_argument("--out-bf16", action="store_true",
                    help="y and dx in bf16 (BIGMAC_FLAG_OUT_BF16) instead of fp32: half the bytes of the two [T, d] results")
    ap.add_argument("--tiles", default="auto", choices=["auto", "large", "small"],
                    help="tuning: force the 256 x 256 workgroup tiles on every expert product that can take them, or forbid them")
    ap.add_argument("--tokens", type=int, default=0, help="override T (decode sweep)")
    ap.add_argument("--forward-only", action="store_true", help="time the inference forward of the workload (no saved block, no backward)")
    ap.add_argument("--no-fused-dispatch", action="store_true",
                    help="dispatch the rows with the copy kernel instead of folding the step into a product (forward-only: "
                         "rows read through the index by the expert-up product; training: rows written through it by "
                         "the descending projection) (BIGMAC_FLAG_NO_FUSED_DISPATCH)")
    ap.add_argument("--order", default="dcca", choices=["dcca", "cdac"])
    ap.add_argument("--cpu-sample", type=int, default=4096, help="tokens of the oracle timing sample (0: skip)")
    ap.add_argument("--no-stage-events", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 512 MiB device copy three times: the kernel of known size that the "
                         "HBM counters (FETCH_SIZE, WRITE_SIZE) of a rocprofv3 --pmc run are scaled by")
    ap.add_argument("--capacity-factor", type=float, default=0.0,
                    help="fixed expert capacity ceil(f T k / N) instead of dropless routing (the paper's training runs: 1.2)")
    ap.add_argument("--aux-alpha", type=float, default=0.0,
                    help="coefficient of the load-balance loss (the paper's training runs: 0.001); 0 = off")
    ap.add_argument("--gather-ceiling", action="store_true",
                    help="only run the library's read-only gather probe (bigmac_gather_probe): what the device moves for the "
                         "combine kernels' access pattern without any write, rows in order and shuffled")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="only time the vendor library's bf16 GEMM (torch.bmm / torch.matmul) at the expert-product shapes of "
                         "--workload with evenly loaded experts: the rate tuned kernels reach on this device at these shapes")
    ap.add_argument("--mfma-peak", action="store_true",
                    help="only time the matrix-core rate probe (register-resident 32x32x16 bf16 MFMAs): the "
                         "achievable dense bf16 peak of this device, printed beside the published one")
    ap.add_argument("--evict-mib", type=int, default=0,
                    help="before every step of the eager pass, overwrite a scratch buffer of this many MiB, so "
                         "that the per-stage times are those of cold caches (512 or more exceeds the 256 MB "
                         "last-level cache); the timed graph replays are not affected")
    ap.add_argument("--no-graph", action="store_true",
                    help="time eager launches instead of replays of the step captured in a HIP graph")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    if args.calibrate_copy:
        n = 512 << 20
        src = torch.full((n,), 1, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "copies": 3}))
        return
    from paper_2502_16927_amd import binding as B
    from paper_2502_16927_amd import synth
    if args.mfma_peak:
        torch.cuda.set_device(0)
        props = torch.cuda.get_device_properties(0)
        sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
        blocks, iters = props.multi_processor_count * 8, 20000
        B.bigmac_mfma_probe(blocks, 100, sink)
        rates = []
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = B.bigmac_mfma_probe(blocks, iters, sink)
            e1.record()
            torch.cuda.synchronize()
            rates.append(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        print(json.dumps({"mfma_probe_tflops": max(rates), "runs": rates, "compute_units": props.multi_processor_count,
                          "clock_mhz": getattr(props, "clock_rate", 0) / 1e3 or None, "published_peak_tflops": PEAK_MFMA_BF16 / 1e12,
                          "probe": "32x32x16 bf16, 4 accumulators per wavefront, %d workgroups x 4 wavefronts" % blocks}))
        return

    def timed_ms(fn, reps=5):
        best = float("inf")
        fn()
        torch.cuda.synchronize()
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1))
        return best

    if args.gather_ceiling:
        torch.cuda.set_device(0)
        rows, row_bytes = 262144, 4096          # the fp32 rows of zipf_stress's combine: 1 GiB
        table = torch.ones(rows * row_bytes // 4, dtype=torch.float32, device="cuda:0")
        sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        rng = np.random.default_rng(1)
        out = {"rows": rows, "row_bytes": row_bytes}
        for name, order in (("in_order", np.arange(rows, dtype=np.int32)), ("shuffled", rng.permutation(rows).astype(np.int32))):
            od = torch.from_numpy(order).to("cuda:0")
            for streaming in (0, 1):
                ms = timed_ms(lambda: B.bigmac_gather_probe(table, od, rows, row_bytes, streaming, sink))
                out["%s_%s_tbps" % (name, "non_temporal" if streaming else "plain")] = round(rows * row_bytes / (ms * 1e-3) / 1e12, 3)
        src = torch.ones(512 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        out["plain_copy_tbps_read_plus_written"] = round(2 * (512 << 20) / (timed_ms(lambda: dst.copy_(src)) * 1e-3) / 1e12, 3)
        print(json.dumps(out))
        return

    wl = synth.WORKLOADS.get(args.workload) or synth.NEXT_WORKLOADS[args.workload]
    if args.vendor_gemm:
        torch.cuda.set_device(0)
        win, hid = (wl.d, wl.r) if args.order == "cdac" else (wl.r, wl.h)
        per = max(8, (wl.T * wl.k // wl.N) // 8 * 8)     # rows per expert, evenly loaded
        a = torch.randn(wl.N, per, win, device="cuda:0", dtype=torch.bfloat16)
        w1 = torch.randn(wl.N, win, hid, device="cuda:0", dtype=torch.bfloat16) * 0.02
        h = torch.randn(wl.N, per, hid, device="cuda:0", dtype=torch.bfloat16)
        w2 = torch.randn(wl.N, hid, win, device="cuda:0", dtype=torch.bfloat16) * 0.02
        flops = 2.0 * wl.N * per * win * hid
        up, down = timed_ms(lambda: torch.bmm(a, w1)), timed_ms(lambda: torch.bmm(h, w2))
        a2, h2 = a.view(wl.N * per, win), h.view(wl.N * per, hid)
        up1, down1 = timed_ms(lambda: torch.matmul(a2, w1[0])), timed_ms(lambda: torch.matmul(h2, w2[0]))
        print(json.dumps({"workload": wl.name, "experts": wl.N, "rows_per_expert": per, "win": win, "hid": hid,
                          "bmm_up_ms": round(up, 4), "bmm_up_tflops": round(flops / up / 1e9, 1),
                          "bmm_down_ms": round(down, 4), "bmm_down_tflops": round(flops / down / 1e9, 1),
                          "one_weight_matmul_up_tflops": round(flops / up1 / 1e9, 1), "one_weight_matmul_down_tflops": round(flops / down1 / 1e9, 1),
                          "note": "plain products, bf16 results, no activation, no saved pre-activation, no ragged groups"}))
        return
    if args.workload == "vanilla_moe":
        args.order = "cdac"   # the vanilla layer is a CDAC-order layer with a wide hidden dimension
    if args.tokens:
        wl = wl.with_T(args.tokens)
    cdac = args.order == "cdac"
    training = wl.backward and not args.forward_only
    dev = "cuda:0"
    torch.cuda.set_device(0)
    data = synth.generate(wl)
    capacity = B.expert_capacity(wl.T, wl.k, wl.N, args.capacity_factor) if args.capacity_factor > 0 else 0
    tile_flag = {"auto": 0, "large": B.FLAG_TILES_LARGE, "small": B.FLAG_TILES_SMALL}[args.tiles]
    dims = B.dims_of(wl, B.ORDER_CDAC if cdac else B.ORDER_DCCA, flags=(B.FLAG_WIRE_BF16 if args.wire_bf16 else 0) | (B.FLAG_OUT_BF16 if args.out_bf16 else 0) | tile_flag | (B.FLAG_NO_FUSED_DISPATCH if args.no_fused_dispatch else 0),
                     capacity=capacity, aux_alpha=args.aux_alpha)
    variant = capacity > 0 or args.aux_alpha > 0 or args.wire_bf16 or args.out_bf16 or args.forward_only or args.no_fused_dispatch   # not the headline configuration
    x = B.to_device(data["x"], wl.dtype, dev)
    dy = B.to_device(data.get("dy"), wl.dtype, dev)
    wg = B.to_device(data["w_gate"], B.F32, dev)
    bias = B.to_device(data["gate_bias"], B.F32, dev)
    if cdac:   # same parameters: the BigMac expert matrices with their roles swapped (needs h == d)
        assert wl.h == wl.d
        w1, w2 = B.to_device(data["w2"], wl.dtype, dev), B.to_device(data["w1"], wl.dtype, dev)
        w_down = w_up = None
        win, hid = wl.d, wl.r
    else:
        w1, w2 = B.to_device(data["w1"], wl.dtype, dev), B.to_device(data["w2"], wl.dtype, dev)
        w_down, w_up = B.to_device(data["w_down"], wl.dtype, dev), B.to_device(data["w_up"], wl.dtype, dev)
        win, hid = wl.r, wl.h
    params = B.make_params(w_down, w_up, wg, bias, w1, w2)
    y = torch.empty((wl.T, wl.d), dtype=torch.float32, device=dev)
    ws = B.alloc_bytes(B.workspace_bytes(dims, B.WS_LAYER_TRAIN if training else B.WS_LAYER_FORWARD), dev)
    saved = B.alloc_bytes(B.workspace_bytes(dims, B.WS_SAVED), dev) if training else None
    if training:
        dx = torch.empty_like(y)
        f32 = lambda *s: torch.empty(s, dtype=torch.float32, device=dev)
        gw = {"d_w_down": None if cdac else f32(wl.d, wl.r), "d_w_up": None if cdac else f32(wl.r, wl.d),
              "d_w_gate": f32(wl.d, wl.N), "d_w1": f32(wl.N, win, hid), "d_w2": f32(wl.N, hid, win)}

    def step():
        B.bigmac_layer_forward(dims, params, x, y, saved, ws)
        if training:
            B.bigmac_layer_backward(dims, params, x, dy, saved, dx, gw["d_w_down"], gw["d_w_up"], gw["d_w_gate"],
                                    gw["d_w1"], gw["d_w2"], ws)

    for _ in range(args.warmup):
        step()
    # Pass 1, eager launches: one pair of HIP events around every stage of every step, on the
    # stream the kernels are launched on (per-stage durations for the roofline).
    tables = [] if args.no_stage_events else [B.StageEvents() for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evict = torch.empty(args.evict_mib << 20, dtype=torch.uint8, device=dev) if args.evict_mib > 0 else None
    for i in range(args.steps):
        if evict is not None:
            evict.fill_(i & 127)
        if tables:
            tables[i].install()
        step()
    torch.cuda.synchronize()
    eager_elapsed = time.perf_counter() - t0
    B.StageEvents.clear()
    # Pass 2, the timed region: the same step (the library only enqueues kernels, no memsets,
    # no synchronisation) captured once in a HIP graph and replayed K times, which removes the
    # host's launch gaps between the ~33 kernels of a step.
    elapsed, timed = eager_elapsed, "eager launches"
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(args.warmup):
            graph.replay()
        block_ms = []
        for b in range(max(1, args.blocks)):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            block_ms.append(dt / args.steps * 1e3)
            if b == 0:
                elapsed, timed = dt, "replays of the step captured in a HIP graph"

    ms_per_step = elapsed / args.steps * 1e3
    work = stage_work(wl, cdac, training, args.wire_bf16)
    stage_ms = {}
    if tables:
        names = [B.stage_name(s) for s in range(B.STAGE_COUNT)]
        fwd_only = {"router_logits", "topk_gate", "descend", "permutation", "dispatch", "expert_up", "expert_down", "combine", "ascend"}
        live = [s for s, n in enumerate(names)
                if (training or n in fwd_only)
                and not (cdac and n in ("descend", "ascend", "bwd_ascend_wgrad", "bwd_descend_wgrad", "bwd_descend_dgrad"))
                and not (not cdac and n == "bwd_output_cast")]
        for tb in tables:
            for s, ms in tb.elapsed_ms(set(live)).items():
                stage_ms[names[s]] = stage_ms.get(names[s], 0.0) + ms / args.steps
    # a dispatch folded into a product has no stage of its own: its bytes are that product's
    folding = B.dispatch_folding(dims, training)
    if folding and "dispatch" in stage_ms:
        del stage_ms["dispatch"]
        if folding == 2:
            kind, flops, nbytes = work["descend"]
            e = 2 if wl.dtype == B.BF16 else 4
            work["descend"] = (kind, flops, nbytes + (wl.T * wl.k - wl.T) * wl.r * e + 4 * wl.T * wl.k)   # k rows written per token, not one
    roofline, stage_roofline = None, {}
    if stage_ms and not capacity:   # with dropped rows the algorithmic work is not the closed form below
        dom = max(stage_ms, key=stage_ms.get)
        kind, flops, nbytes = work[dom]
        roofline = roofline_of(dom, kind, flops, nbytes, stage_ms[dom] * 1e-3)
        if not args.tokens and not variant:
            measured = MEASURED_TRAFFIC.get((wl.name, args.order), {})
            roofline["traffic"] = sum(measured[dom]) * 1048576 if dom in measured else None
            roofline["traffic_source"] = measured.get("source") if dom in measured else None
        # every stage against both of its rooflines: matrix (or fp32 vector) rate and HBM bytes
        for n, ms in stage_ms.items():
            kind, flops, nbytes = work[n]
            peak_f = PEAK_ALU_F32 if kind == "alu" else PEAK_MFMA_BF16
            stage_roofline[n] = {"bound": roofline_of(n, kind, flops, nbytes, ms * 1e-3)["bound"],
                                 "flop_frac": round(flops / (ms * 1e-3) / peak_f, 4) if flops and kind != "hbm" else None,
                                 "hbm_frac": round(nbytes / (ms * 1e-3) / PEAK_HBM, 4)}
    fwd_flops = B.forward_matrix_flops(dims)
    out = {
        "metric": "BigMac MoE layer tokens/sec fwd+bwd (1 GPU)" if training else "BigMac MoE layer tokens/sec fwd (1 GPU)",
        "value": wl.T / (elapsed / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == B.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "order": args.order, "T": wl.T, "d": wl.d, "r": wl.r, "N": wl.N, "k": wl.k,
                   "h": wl.h, "pass": "fwd+bwd" if training else "fwd",
                   **({"capacity_factor": args.capacity_factor, "capacity": capacity} if capacity else {}),
                   **({"aux_alpha": args.aux_alpha} if args.aux_alpha > 0 else {}),
                   **({"wire": "bf16"} if args.wire_bf16 else {}), **({"out": "bf16"} if args.out_bf16 else {}), **({"tiles": args.tiles} if args.tiles != "auto" else {}),
                   **({"dispatch": "separate kernel"} if args.no_fused_dispatch else {})},
        "timed": timed,
        **({"block_ms_per_step": [round(v, 4) for v in block_ms], "block_ms_median": round(sorted(block_ms)[len(block_ms) // 2], 4),
            "block_ms_min": round(min(block_ms), 4)} if not args.no_graph else {}),
        "eager_ms_per_step": eager_elapsed / args.steps * 1e3,
        "roofline": roofline,
        "matrix_tflops": fwd_flops * (3 if training else 1) / (elapsed / args.steps) / 1e12,
        "permute_bytes_per_step": B.permute_bytes(dims) * (1.0 if training else 0.5),
        "dispatch": {0: "copy kernel", 1: "folded into the expert-up product (rows read through src_of)",
                     2: "folded into the descending projection (rows written through slot_of)"}[folding],
        "stage_ms": {n: round(v, 4) for n, v in stage_ms.items()},
        "stage_roofline": stage_roofline,
        "stage_sum_ms": round(sum(stage_ms.values()), 4),
    }
    if args.evict_mib > 0:
        out["stage_ms_caches"] = "cold: %d MiB overwritten before every eager step" % args.evict_mib
        if stage_ms:   # the permutes against their compulsory bytes
            out["permute_gbps_cold"] = {n: round(work[n][2] / (stage_ms[n] * 1e-3) / 1e9, 1)
                                        for n in ("dispatch", "combine", "bwd_combine", "bwd_dispatch") if n in stage_ms}
    if args.cpu_sample > 0 and not cdac and not variant:
        out["cpu_baseline"] = cpu_baseline(wl, data, args.cpu_sample, training)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
