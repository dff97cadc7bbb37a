#!/usr/bin/env python3
"""ConvAttn forward benchmark on one MI355X.

A step is one esc_convattn_forward call with the kernel estimator (GAP, estimator,
fused LK+DK depth-wise convolution, pass-through copy) on one batch of a
synthetic workload (paper_2503_06671_amd/workloads.py).  Default workload: the
720p-output x4 feature map (1x64x180x320 fp32, C_a=16, Ks=13).

Inputs are resident in HBM before timing.  Steps rotate over enough distinct
(x, out) buffer pairs to exceed the on-chip caches (--rotate-bytes), so the
figure is an HBM figure, not a cache figure; --warm-cache times a single pair.
The K timed steps are captured into one HIP graph and replayed (so the host's
launch rate does not bound a few-microsecond step); --eager times plain calls.

Prints ONE JSON line.
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

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, vendor figure
FP32_VECTOR_PEAK_TFLOPS = 157.3  # 256 CU x 2.4 GHz x 256 flop/clk

# HBM bytes per launch of the forward kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# scaled against a plain copy of known size (see the summaries under profiles/).
MEASURED_TRAFFIC_BYTES = {
    "cfg1_hd_x4_180x320_f32": 29.92e6,  # profiles/forward_kernel_ks13_f32_cfg1_180x320.txt
    "cfg4_1080p_x2_540x960_f32_ks13": 288.0e6,  # profiles/forward_kernel_ks13_f32_cfg4_540x960.txt
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--config", type=int, default=1, help="workload index 0..4; 5 = the large-model point (C = 192, C_a = 48, h = 24)")
    ap.add_argument("--ks", type=int, default=None, help="kernel size for workload 4")
    ap.add_argument("--rotate-bytes", type=float, default=1.0e9)
    ap.add_argument("--warm-cache", action="store_true", help="one buffer pair (cache-resident)")
    ap.add_argument("--eager", action="store_true", help="time plain calls instead of a graph replay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def cpu_baseline(wl):
    """The oracle as it stands, whole forward on the same workload, best of 3."""
    from oracle import esc_oracle
    esc_oracle.build()
    best = float("inf")
    reps = 0
    t_all = time.perf_counter()
    while reps < 3 or (time.perf_counter() - t_all < 8.0 and reps < 20):
        t0 = time.perf_counter()
        esc_oracle.forward_workload(wl, want_out=True)
        best = min(best, time.perf_counter() - t0)
        reps += 1
    return {"value": wl.pixels / best / 1e6, "unit": "Mpixel/s", "cores": esc_oracle.threads(),
            "kind": "oracle", "ms_per_step": best * 1e3,
            "sample": f"whole workload {wl.name}, full forward, best of {reps} runs"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path needs no collective; "
              "see DESIGN.md for how it would shard); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2503_06671_amd import binding, workloads as wk

    binding.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.config == 5:
        wl = wk.make_large_model()
    else:
        wl = wk.make_config(args.config, args.ks) if args.config == 4 else wk.make_config(args.config)
    es = wl.elem_bytes
    b_alg = 2.0 * wl.N * wl.C * wl.H * wl.W * es            # read x once, write out once
    f_alg = 2.0 * wl.Ks * wl.Ks * wl.N * wl.Ca * wl.H * wl.W  # merged-kernel tap count
    pairs = 1 if args.warm_cache else max(2, int(np.ceil(args.rotate_bytes / b_alg)))

    if wl.dtype == wk.F32:
        x0 = torch.from_numpy(wl.x).cuda()
    else:
        x0 = torch.from_numpy(wl.x.view(np.int16)).cuda().view(torch.bfloat16)
    xs = [x0] + [x0.clone() for _ in range(pairs - 1)]
    outs = [torch.empty_like(x0) for _ in range(pairs)]
    lk = torch.from_numpy(wl.lk).cuda()
    def dev(a):
        return None if a is None else torch.from_numpy(a).cuda()

    gen = binding.GenParams(dev(wl.w_up), dev(wl.b_up), wl.hidden, dev(wl.w_down), dev(wl.b_down))
    ws = binding.new_workspace(wl.N, wl.Ca, wl.H, wl.W)
    stream = torch.cuda.Stream()

    def step(i):
        binding.convattn_forward(xs[i % pairs], wl.Ca, lk, ws, gen=gen, out=outs[i % pairs], stream=stream)

    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            step(i)
    torch.cuda.synchronize()

    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    mode = "eager"
    if not args.eager:
        mode = "hipgraph"
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(args.steps):
                step(i)
        with torch.cuda.stream(stream):
            graph.replay()                      # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            ev0.record(stream)
            graph.replay()
            ev1.record(stream)
        torch.cuda.synchronize()
    else:
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            ev0.record(stream)
            for i in range(args.steps):
                step(i)
            ev1.record(stream)
        torch.cuda.synchronize()
    ms_total = ev0.elapsed_time(ev1)
    ms_step = ms_total / args.steps

    # spot check of the last buffers against the first (same input => same bits), and no
    # bounded wait inside the kernel may have expired
    assert torch.equal(outs[0], outs[(args.steps - 1) % pairs]), "rotating buffers disagree"
    assert binding.workspace_errors(ws, stream) == 0, "a wait inside the kernel expired"

    sec = ms_step * 1e-3
    res = {
        "metric": "convattn_fwd_mpixel_per_s",
        "value": wl.pixels / sec / 1e6,
        "unit": "Mpixel/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wk.DTYPE_NAMES[wl.dtype],
        "data": "synthetic",
        "config": {"workload": wl.name, "N": wl.N, "C": wl.C, "C_a": wl.Ca, "H": wl.H, "W": wl.W,
                   "Ks": wl.Ks, "launch": mode, "buffer_pairs": pairs,
                   "cache": "warm" if args.warm_cache else "rotating"},
        "hbm_gbps_algorithmic": b_alg / sec / 1e9,
        "valu_tflops": f_alg / sec / 1e12,
        # one step is one launch of the single forward kernel, so the per-launch duration is
        # the HIP-event time of the timed region divided by the number of launches
        "roofline": {
            "bound": "hbm",
            "kernel": f"forward_kernel<{wl.Ks}, RY, {'float' if wl.dtype == wk.F32 else 'bf16'}> (the only kernel of a step)",
            "achieved": b_alg / sec / 1e9,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": b_alg / sec / 1e9 / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name) if not args.warm_cache else None,
            "algorithmic_bytes": b_alg,
            "kernel_us": ms_step * 1e3,
            "alu_tflops": f_alg / sec / 1e12,
            "alu_frac_of_fp32_vector_peak": f_alg / sec / 1e12 / FP32_VECTOR_PEAK_TFLOPS,
        },
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
