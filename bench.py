#!/usr/bin/env python3
"""ConvAttn forward benchmark on one MI355X.

A step is one esc_convattn_forward call with the kernel estimator (GAP, estimator,
fused LK+DK depth-wise convolution, pass-through copy) on one batch of a
synthetic workload (paper_2503_06671_amd/workloads.py).  Default workload: the
720p-output x4 feature map (1x64x180x320 fp32, C_a=16, Ks=13).

Inputs are resident in HBM before timing.  Steps rotate over enough distinct
(x, out) buffer pairs to exceed the on-chip caches (--rotate-bytes), so the
figure is an HBM figure, not a cache figure; --warm-cache times a single pair.
After W untimed warm-up steps the K timed steps are captured into one HIP graph
(so the host's launch rate does not bound a few-microsecond step) and the graph
is replayed `config.replays` times, each replay bracketed by HIP events on the
launch stream; `ms_per_step` is the median over the replays (clocks need a few
milliseconds of work to settle, which a single short replay does not give them).
--eager times plain calls instead.  Also reported: the latency of one call after a
device synchronisation, the same timing for the other benchmark workloads
(`all_workloads`), and two floors measured in the same process with the library's
own calls: a pure copy of the same tensors (C_a = 0) and a call with nothing to do.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0                 # MI355X HBM3E, vendor figure
FP32_VECTOR_PEAK_TFLOPS = 157.3       # 256 CU x 2.4 GHz x 256 flop/clk (counts the packed fp32 forms)
FP32_VECTOR_UNPACKED_TFLOPS = 78.6    # the same without them (they are switched off in this build)
FP32_FMA_MEASURED_TFLOPS = 118.0      # 0.375 plain FMAs per clock and SIMD, the best rate measured on this chip


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=2000)
    ap.add_argument("--config", type=int, default=1,
                    help="workload index 0..4; 5 = the large-model point (C = 192, C_a = 48, h = 24)")
    ap.add_argument("--ks", type=int, default=None, help="kernel size for workload 4")
    ap.add_argument("--rotate-bytes", type=float, default=1.0e9)
    ap.add_argument("--replays", type=int, default=0, help="timed graph replays (0 = at least 50 and 20000 launches)")
    ap.add_argument("--warm-cache", action="store_true", help="one buffer pair (cache-resident)")
    ap.add_argument("--eager", action="store_true", help="time plain calls instead of graph replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-workloads", action="store_true", help="skip the other benchmark workloads")
    ap.add_argument("--no-floors", action="store_true", help="skip the copy-only and empty-call floors")
    ap.add_argument("--fused", action="store_true",
                    help="time esc_convattn_fused_forward (the module with Conv_fuse, Eq. 4 line 4) instead")
    ap.add_argument("--dense", action="store_true",
                    help="time esc_convattn_dense_forward (dense Ks x Ks x C_a x C_a large kernel of the paper's main variants) instead")
    ap.add_argument("--backward", action="store_true",
                    help="time esc_convattn_backward (gradients of the depth-wise forward) instead")
    ap.add_argument("--ffn", action="store_true",
                    help="time esc_convffn_forward (ConvFFN of Eq. 3 line 3, hidden width 2 C) instead")
    ap.add_argument("--res-step", action="store_true",
                    help="time the whole residual step of Eq. 3 line 3 (esc_residual_step_forward: ConvFFN, then "
                         "the fused module on its output with residual = the step's input)")
    ap.add_argument("--lkc", action="store_true", help="with --fused: LK^c in front of the depth-wise kernels (Eq. 5)")
    ap.add_argument("--residual", action="store_true", help="with --fused: add the residual of Eq. 3 line 3")
    return ap.parse_args()


def source_hash() -> str:
    """Hash of the kernel sources: a profile summary applies to the build it was taken from."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2503_06671_amd", "csrc")
    for f in sorted(glob.glob(os.path.join(csrc, "*.hip")) + glob.glob(os.path.join(csrc, "*.hpp"))):
        h.update(os.path.basename(f).encode())
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def profiled_traffic(workload_name: str):
    """HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary under
    profiles/ for this workload - if that summary was taken from the current kernel sources
    (the summaries carry the source hash), else None."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        text = open(path).read()
        m_w = re.search(r"^workload:\s*(\S+)", text, re.M)
        m_t = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
        m_h = re.search(r"^kernel_source_sha16:\s*([0-9a-f]+)", text, re.M)
        if m_w and m_t and m_h and m_w.group(1) == workload_name:
            if m_h.group(1) == source_hash():
                return float(m_t.group(1)), os.path.relpath(path, ROOT)
            return None, os.path.relpath(path, ROOT) + " (taken from other kernel sources: not used)"
    return None, None


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl):
    """The oracle as it stands (float64 accumulators, never tuned), whole forward on the same
    workload: best of several runs on all threads, and best of 3 on one thread."""
    from oracle import esc_oracle
    esc_oracle.build()
    nthreads = esc_oracle.threads()
    best = float("inf")
    reps = 0
    t_all = time.perf_counter()
    while reps < 3 or (time.perf_counter() - t_all < 8.0 and reps < 20):
        t0 = time.perf_counter()
        esc_oracle.forward_workload(wl, want_out=True)
        best = min(best, time.perf_counter() - t0)
        reps += 1
    esc_oracle.set_threads(1)
    best1 = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        esc_oracle.forward_workload(wl, want_out=True)
        best1 = min(best1, time.perf_counter() - t0)
    esc_oracle.set_threads(nthreads)
    return {"value": wl.pixels / best / 1e6, "unit": "Mpixel/s", "cores": nthreads,
            "kind": "oracle", "ms_per_step": best * 1e3, "ms_per_step_1thread": best1 * 1e3,
            "cpu_model": cpu_model(), "host_cpus": os.cpu_count(),
            "sample": f"whole workload {wl.name}, full forward, best of {reps} runs on {nthreads} threads "
                      f"and best of 3 on one thread"}


BF16_MFMA_PEAK_TFLOPS = 2500.0        # dense bf16 matrix-core peak


def taps_on_matrix_cores(wl) -> bool:
    """bf16 storage with Ks <= 17: the library runs the depth-wise taps as bf16 matrix
    instructions (fp32 accumulation), so their roof is the bf16 matrix peak."""
    return wl.elem_bytes == 2 and wl.Ks <= 17


def roofline_of(wl, sec):
    """Which roof bounds this workload (HBM at 8 TB/s, or the units the taps run on: the fp32
    vector units at 157.3 TFLOP/s, for bf16 storage with Ks <= 17 the bf16 matrix cores at
    2.5 PFLOP/s) and the fraction of it reached; the fractions against the other ceilings ride along."""
    b_alg = 2.0 * wl.N * wl.C * wl.H * wl.W * wl.elem_bytes   # read x once, write out once
    f_alg = 2.0 * wl.Ks * wl.Ks * wl.N * wl.Ca * wl.H * wl.W  # merged-kernel tap count
    t_hbm = b_alg / (HBM_PEAK_GBS * 1e9)
    on_mfma = taps_on_matrix_cores(wl)
    alu_peak = BF16_MFMA_PEAK_TFLOPS if on_mfma else FP32_VECTOR_PEAK_TFLOPS
    t_alu = f_alg / (alu_peak * 1e12)
    gbs, tfl = b_alg / sec / 1e9, f_alg / sec / 1e12
    if t_hbm >= t_alu:
        r = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}
    else:
        r = {"bound": "mfma" if on_mfma else "alu", "achieved": tfl, "peak": alu_peak, "unit": "TFLOP/s",
             "frac": tfl / alu_peak}
    r.update({
        "algorithmic_bytes": b_alg, "algorithmic_flops": f_alg,
        "hbm_gbps": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS,
        "alu_tflops": tfl, "frac_of_fp32_vector_peak": tfl / FP32_VECTOR_PEAK_TFLOPS,
        "frac_of_fp32_vector_peak_unpacked": tfl / FP32_VECTOR_UNPACKED_TFLOPS,
        "frac_of_fp32_fma_rate_measured": tfl / FP32_FMA_MEASURED_TFLOPS,
        # the roof itself with the unpacked ceiling: max(HBM time, ALU time at 78.6 TFLOP/s) / measured
        "frac_of_roof_unpacked": max(t_hbm, f_alg / (FP32_VECTOR_UNPACKED_TFLOPS * 1e12)) / sec,
    })
    return r


FP32_MFMA_PEAK_TFLOPS = 157.3         # dense fp32 matrix-core peak


def fused_roofline_of(wl, sec, lkc, residual):
    """The fused call: x read once (plus the residual), out written once; the depth-wise taps on
    the vector units, Conv_fuse (and LK^c) on the matrix cores in fp32 - with bf16 storage both
    on the bf16 matrix cores (taps: Ks <= 17), whose peak is then the one that counts."""
    P = wl.N * wl.H * wl.W
    b_alg = (3.0 if residual else 2.0) * P * wl.C * wl.elem_bytes
    f_vec = 2.0 * wl.Ks * wl.Ks * P * wl.Ca
    f_mat = 2.0 * wl.C * wl.C * P + (2.0 * wl.Ca * wl.Ca * P if lkc else 0.0)
    taps_peak = BF16_MFMA_PEAK_TFLOPS if taps_on_matrix_cores(wl) else FP32_VECTOR_PEAK_TFLOPS
    mat_peak = BF16_MFMA_PEAK_TFLOPS if wl.elem_bytes == 2 else FP32_MFMA_PEAK_TFLOPS
    t = {"hbm": b_alg / (HBM_PEAK_GBS * 1e9), "alu": f_vec / (taps_peak * 1e12), "mfma": f_mat / (mat_peak * 1e12)}
    bound = max(t, key=t.get)
    ach = {"hbm": b_alg / sec / 1e9, "alu": f_vec / sec / 1e12, "mfma": f_mat / sec / 1e12}[bound]
    peak = {"hbm": HBM_PEAK_GBS, "alu": taps_peak, "mfma": mat_peak}[bound]
    return {"bound": bound, "achieved": ach, "peak": peak, "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
            "frac": ach / peak, "algorithmic_bytes": b_alg, "algorithmic_flops_vector": f_vec,
            "algorithmic_flops_matrix": f_mat, "hbm_gbps": b_alg / sec / 1e9, "alu_tflops": f_vec / sec / 1e12,
            "mfma_tflops": f_mat / sec / 1e12}


def dense_roofline_of(wl, sec):
    """The dense-LK call: same bytes as the depth-wise forward; the C_a x C_a x Ks x Ks contraction on the
    matrix cores, DK's nine taps on the vector units.  With up to 16 channels the contraction runs on the
    bf16 instructions: bf16 storage with every weight as two bf16 terms (two instructions per product
    block), fp32 storage (Ks <= 13) with every value and weight as three exact bf16 terms (six
    instructions per product block).  What bounds such a kernel is the instructions it issues at the
    bf16 peak: `achieved` counts those (`terms_per_product` times the algorithmic flops, which hold
    each product once and are reported beside it, also against the fp32 matrix peak).  Otherwise
    fp32 instructions at the fp32 matrix peak."""
    P = wl.N * wl.H * wl.W
    b_alg = 2.0 * P * wl.C * wl.elem_bytes
    f_mat = 2.0 * wl.Ks * wl.Ks * wl.Ca * wl.Ca * P
    on_bf16 = wl.Ca <= 16 and (wl.elem_bytes == 2 or wl.Ks <= 13)
    mat_peak = BF16_MFMA_PEAK_TFLOPS if on_bf16 else FP32_MFMA_PEAK_TFLOPS
    issued = (2.0 if wl.elem_bytes == 2 else 6.0) if on_bf16 else 1.0
    t_hbm, t_mat = b_alg / (HBM_PEAK_GBS * 1e9), issued * f_mat / (mat_peak * 1e12)
    if t_hbm >= t_mat:
        r = {"bound": "hbm", "achieved": b_alg / sec / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s"}
    else:
        r = {"bound": "mfma", "achieved": issued * f_mat / sec / 1e12, "peak": mat_peak, "unit": "TFLOP/s"}
    r["frac"] = r["achieved"] / r["peak"]
    r.update({"algorithmic_bytes": b_alg, "algorithmic_flops_matrix": f_mat, "terms_per_product": issued,
              "matrix_instructions": "bf16" if on_bf16 else "fp32", "hbm_gbps": b_alg / sec / 1e9,
              "mfma_tflops": f_mat / sec / 1e12, "mfma_issued_tflops": issued * f_mat / sec / 1e12,
              "algorithmic_frac_of_fp32_mfma_peak": f_mat / sec / 1e12 / FP32_MFMA_PEAK_TFLOPS,
              "algorithmic_frac_of_bf16_mfma_peak": f_mat / sec / 1e12 / BF16_MFMA_PEAK_TFLOPS, "alu_tflops": 0.0})
    return r


def backward_roofline_of(wl, sec):
    """The backward call: x and grad_out read once, grad_x written once (3 tensors); two passes of
    2 Ks^2 flops per attention pixel: the correlation (on the bf16 matrix cores for Ks <= 15 - fp32
    values as three exact bf16 terms each, nine instructions per product block, which the algorithmic
    count does not include - else on the vector units) and the input gradient (the forward kernel: the
    vector units, or the bf16 matrix cores where the forward's taps run there)."""
    P = wl.N * wl.H * wl.W
    b_alg = 3.0 * P * wl.C * wl.elem_bytes
    f_alg = 4.0 * wl.Ks * wl.Ks * P * wl.Ca
    f_vec = (0.0 if wl.Ks <= 15 else f_alg / 2.0) + (0.0 if taps_on_matrix_cores(wl) else f_alg / 2.0)
    f_mat = f_alg - f_vec
    t = {"hbm": b_alg / (HBM_PEAK_GBS * 1e9), "alu": f_vec / (FP32_VECTOR_PEAK_TFLOPS * 1e12),
         "mfma": f_mat / (BF16_MFMA_PEAK_TFLOPS * 1e12)}
    bound = max(t, key=t.get)
    ach = {"hbm": b_alg / sec / 1e9, "alu": f_vec / sec / 1e12, "mfma": f_mat / sec / 1e12}[bound]
    peak = {"hbm": HBM_PEAK_GBS, "alu": FP32_VECTOR_PEAK_TFLOPS, "mfma": BF16_MFMA_PEAK_TFLOPS}[bound]
    return {"bound": bound, "achieved": ach, "peak": peak, "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
            "frac": ach / peak, "algorithmic_bytes": b_alg, "algorithmic_flops": f_alg, "hbm_gbps": b_alg / sec / 1e9,
            "alu_tflops": f_vec / sec / 1e12, "mfma_tflops": f_mat / sec / 1e12}


def ffn_roofline_of(wl, sec, with_module):
    """ConvFFN (hidden width 2 C): x read once, out written once; the two point-wise layers on the
    matrix cores (fp32 instructions for fp32 storage; bf16 storage: bf16 instructions, two per product
    block because every weight is two bf16 terms - `achieved` counts those), the 3 x 3 branch and the
    two GELUs per hidden element on the vector units.  with_module: the whole residual step, the fused module's work and bytes added
    (the tensor between the two calls is written and read once more: it is an output and an input)."""
    P = wl.N * wl.H * wl.W
    Ch = 2 * wl.C
    b_alg = 2.0 * P * wl.C * wl.elem_bytes
    f_mat = 4.0 * wl.C * Ch * P
    # the branch's nine multiply-adds and two GELUs per hidden element; an erf-form GELU is priced at the
    # operation count of the evaluation the kernels use (rational erf: a reciprocal, an exponential,
    # nine multiply-adds, six other operations): 30 flops
    f_vec = (18.0 + 2.0 * 30.0) * Ch * P
    if with_module:
        b_alg += 3.0 * P * wl.C * wl.elem_bytes
        f_mat += 2.0 * wl.C * wl.C * P
        f_taps = 2.0 * wl.Ks * wl.Ks * P * wl.Ca
    else:
        f_taps = 0.0
    issued = 2.0 if wl.elem_bytes == 2 else 1.0
    mat_peak = BF16_MFMA_PEAK_TFLOPS if wl.elem_bytes == 2 else FP32_MFMA_PEAK_TFLOPS
    taps_peak = BF16_MFMA_PEAK_TFLOPS if taps_on_matrix_cores(wl) else FP32_VECTOR_PEAK_TFLOPS
    t = {"hbm": b_alg / (HBM_PEAK_GBS * 1e9), "mfma": issued * f_mat / (mat_peak * 1e12),
         "alu": f_vec / (FP32_VECTOR_PEAK_TFLOPS * 1e12) + f_taps / (taps_peak * 1e12)}
    bound = max(t, key=t.get)
    ach = {"hbm": b_alg / sec / 1e9, "mfma": issued * f_mat / sec / 1e12, "alu": (f_vec + f_taps) / sec / 1e12}[bound]
    peak = {"hbm": HBM_PEAK_GBS, "mfma": mat_peak, "alu": FP32_VECTOR_PEAK_TFLOPS}[bound]
    return {"bound": bound, "achieved": ach, "peak": peak, "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
            "frac": t[bound] / sec, "algorithmic_bytes": b_alg, "algorithmic_flops_matrix": f_mat,
            "algorithmic_flops_vector": f_vec + f_taps, "terms_per_product": issued, "hidden_channels": Ch,
            "hbm_gbps": b_alg / sec / 1e9, "mfma_tflops": f_mat / sec / 1e12, "alu_tflops": (f_vec + f_taps) / sec / 1e12}


class Runner:
    """Device buffers of one workload and the timing protocol."""

    def __init__(self, wl, rotate_bytes, warm_cache, ca=None, fused=None, dense=False, backward=False, ffn=None):
        import numpy as np
        import torch
        from paper_2503_06671_amd import binding, workloads as wk
        self.torch, self.binding, self.wl = torch, binding, wl
        self.ca = wl.Ca if ca is None else ca
        b_alg = 2.0 * wl.N * wl.C * wl.H * wl.W * wl.elem_bytes
        self.pairs = 1 if warm_cache else max(2, int(np.ceil(rotate_bytes / b_alg)))
        if wl.dtype == wk.F32:
            x0 = torch.from_numpy(wl.x).cuda()
        else:
            x0 = torch.from_numpy(wl.x.view(np.int16)).cuda().view(torch.bfloat16)
        self.xs = [x0] + [x0.clone() for _ in range(self.pairs - 1)]
        self.outs = [torch.empty_like(x0) for _ in range(self.pairs)]
        self.lk = torch.from_numpy(wl.lk).cuda()

        def dev(a):
            return None if a is None else torch.from_numpy(a).cuda()

        self.gen = None
        if self.ca > 0:
            self.gen = binding.GenParams(dev(wl.w_up), dev(wl.b_up), wl.hidden, dev(wl.w_down), dev(wl.b_down))
        self.fused = fused
        self.dense = dense
        self.backward = backward
        if backward:
            self.gos = [torch.randn_like(x0) for _ in range(self.pairs)]   # seeded by torch's default generator below
            self.ws = binding.new_backward_workspace(wl.N, self.ca, wl.H, wl.W, wl.Ks, wl.hidden)
            self.grads = None   # the first call allocates the parameter-gradient buffers, later calls reuse them
        elif dense:
            # seeded dense large kernel [C_a, C_a, Ks, Ks] ~ N(0, 1 / (Ks^2 C_a))
            rng = np.random.default_rng(2000 + wl.Ks)
            self.lk_dense = dev((rng.standard_normal((wl.Ca, wl.Ca, wl.Ks, wl.Ks)) / (wl.Ks * np.sqrt(wl.Ca))).astype(np.float32))
            self.ws = binding.new_dense_workspace(wl.N, self.ca, wl.H, wl.W, wl.Ks)
        elif fused is None:
            self.ws = binding.new_workspace(wl.N, self.ca, wl.H, wl.W)
        else:
            # seeded point-wise weights: Conv_fuse [C,C] ~ N(0, 1/C) with a small bias, LK^c [C_a,C_a] ~ N(0, 1/C_a)
            rng = np.random.default_rng(1000 + wl.C)
            self.w_fuse = dev((rng.standard_normal((wl.C, wl.C)) / np.sqrt(wl.C)).astype(np.float32))
            self.b_fuse = dev((rng.standard_normal(wl.C) * 0.1).astype(np.float32))
            self.lk_c = dev((rng.standard_normal((wl.Ca, wl.Ca)) / np.sqrt(wl.Ca)).astype(np.float32)) if fused["lkc"] else None
            self.res = [torch.randn_like(x0) for _ in range(self.pairs)] if fused["residual"] else None
            self.ws = binding.new_fused_workspace(wl.N, self.ca, wl.H, wl.W, x0.dtype, fused["lkc"])
        self.ffn = ffn   # None, "ffn" (ConvFFN alone) or "step" (ConvFFN, then the fused module with the residual)
        if ffn is not None:
            fp = wk.make_ffn_params(3000 + wl.C, wl.C, 2 * wl.C)
            self.ffn_p = {k: dev(v) for k, v in fp.items()}
            self.ffn_ws = binding.new_convffn_workspace(wl.N, 2 * wl.C, wl.H, wl.W, x0.dtype)
            if ffn == "step":   # esc_residual_step_forward: one workspace, which begins with the fused call's
                self.ws = binding.new_residual_step_workspace(wl.N, wl.C, wl.H, wl.W, self.ca, 2 * wl.C, x0.dtype,
                                                              bool(fused and fused["lkc"]))
        self.stream = torch.cuda.Stream()

    def step(self, i):
        k = i % self.pairs
        if self.ffn is not None:
            p = self.ffn_p
            if self.ffn == "step":
                self.binding.residual_step_forward(
                    self.xs[k], p["w1"], p["k"], p["w2"], self.ca, self.lk, self.w_fuse, self.ws, b1=p["b1"],
                    b_dw=p["bk"], b2=p["b2"], lk_c=self.lk_c, gen=self.gen, b_fuse=self.b_fuse, out=self.outs[k],
                    stream=self.stream)
            else:
                self.binding.convffn_forward(self.xs[k], p["w1"], p["k"], p["w2"], self.ffn_ws, b1=p["b1"], b_dw=p["bk"],
                                             b2=p["b2"], out=self.outs[k], stream=self.stream)
            return
        if self.backward:
            g = dict(self.grads or {})
            g["grad_x"] = self.outs[k]
            self.grads = self.binding.convattn_backward(self.xs[k], self.gos[k], self.ca, self.lk, self.ws, gen=self.gen,
                                                        grads=g, stream=self.stream)
            return
        if self.dense:
            self.binding.convattn_dense_forward(self.xs[k], self.ca, self.lk_dense, self.ws, gen=self.gen, out=self.outs[k],
                                                stream=self.stream)
            return
        if self.fused is not None:
            self.binding.convattn_fused_forward(
                self.xs[k], self.ca, self.lk, self.w_fuse, self.ws, b_fuse=self.b_fuse, lk_c=self.lk_c,
                residual=None if self.res is None else self.res[k], gen=self.gen, out=self.outs[k], stream=self.stream)
            return
        self.binding.convattn_forward(self.xs[k], self.ca, self.lk, self.ws, gen=self.gen, out=self.outs[k],
                                      stream=self.stream)

    def time(self, steps, warmup, replays, eager=False):
        """Median (and spread) of the per-step time over `replays` timed regions of `steps` launches."""
        torch = self.torch
        with torch.cuda.stream(self.stream):
            for i in range(warmup):
                self.step(i)
        torch.cuda.synchronize()
        graph = None
        if not eager:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=self.stream):
                for i in range(steps):
                    self.step(i)
            with torch.cuda.stream(self.stream):
                graph.replay()                  # untimed: the first replay uploads the graph
            torch.cuda.synchronize()
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
        with torch.cuda.stream(self.stream):
            for e0, e1 in pairs:
                e0.record(self.stream)
                if graph is not None:
                    graph.replay()
                else:
                    for i in range(steps):
                        self.step(i)
                e1.record(self.stream)
        torch.cuda.synchronize()
        per = sorted(e0.elapsed_time(e1) / steps for e0, e1 in pairs)
        first = pairs[0][0].elapsed_time(pairs[0][1]) / steps
        assert self.binding.workspace_errors(self.ws, self.stream) == 0, "a wait inside the kernel expired"
        return {"median": per[len(per) // 2], "min": per[0], "max": per[-1], "first": first}

    def single_call_latency_us(self, reps=25):
        """One call after a device synchronisation, event to event; median of `reps`."""
        torch = self.torch
        lat = []
        for i in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            with torch.cuda.stream(self.stream):
                e0.record(self.stream)
                self.step(i)
                e1.record(self.stream)
            torch.cuda.synchronize()
            lat.append(e0.elapsed_time(e1) * 1e3)
        lat.sort()
        return lat[len(lat) // 2]


def replays_for(steps, asked):
    if asked > 0:
        return asked
    return max(50, -(-20000 // steps))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (the path shards over images, channels or row "
              "bands without a collective, but only one GPU is built and timed); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_06671_amd import binding, workloads as wk

    binding.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.config == 5:
        wl = wk.make_large_model()
    else:
        wl = wk.make_config(args.config, args.ks) if args.config == 4 else wk.make_config(args.config)
    replays = replays_for(args.steps, args.replays)

    fused = {"lkc": args.lkc, "residual": args.residual} if args.fused else None
    ffn = "step" if args.res_step else "ffn" if args.ffn else None
    if ffn == "step":
        fused = {"lkc": args.lkc, "residual": False}   # (the residual is the step's input, not a tensor of its own)
    torch.manual_seed(7)
    run = Runner(wl, args.rotate_bytes, args.warm_cache, fused=fused, dense=args.dense, backward=args.backward, ffn=ffn)
    t = run.time(args.steps, args.warmup, replays, eager=args.eager)
    ms_step = t["median"]
    # spot check of the last buffers against the first (same input => same bits)
    if not args.residual and not args.backward:
        assert torch.equal(run.outs[0], run.outs[(args.steps - 1) % run.pairs]), "rotating buffers disagree"
    latency_us = run.single_call_latency_us()

    floors = None
    if not args.no_floors and fused is None and not args.dense and not args.backward and ffn is None:
        # the library's own pure copy (C_a = 0) on the same tensors and rotation, and a call
        # with nothing to do (1 x 1 x 1 x 1, C_a = 0): what is left above them is the method's
        copy_t = Runner(wl, args.rotate_bytes, args.warm_cache, ca=0).time(args.steps, min(args.warmup, 200), replays,
                                                                          eager=args.eager)
        tiny = wk.make_random(0, 1, 1, 1, 1, 0, 1)
        empty_t = Runner(tiny, 1.0, True).time(args.steps, min(args.warmup, 200), replays, eager=args.eager)
        floors = {"copy_only_us": copy_t["median"] * 1e3, "empty_call_us": empty_t["median"] * 1e3,
                  "what": "esc_convattn_forward with C_a = 0 on the same tensors and rotation; the same on a "
                          "1x1x1x1 tensor; medians over the same number of replays"}
    del run

    sec = ms_step * 1e-3
    wl_name = wl.name
    if ffn is not None:
        wl_name += "_convffn" if ffn == "ffn" else "_residual_step" + ("_lkc" if args.lkc else "")
        roof = ffn_roofline_of(wl, sec, ffn == "step")
    elif fused is not None:
        wl_name += "_fused" + ("_lkc" if args.lkc else "") + ("_res" if args.residual else "")
        roof = fused_roofline_of(wl, sec, args.lkc, args.residual)
    elif args.dense:
        wl_name += "_dense"
        roof = dense_roofline_of(wl, sec)
    elif args.backward:
        wl_name += "_backward"
        roof = backward_roofline_of(wl, sec)
    else:
        roof = roofline_of(wl, sec)
    traffic, traffic_src = (None, None) if args.warm_cache else profiled_traffic(wl_name)
    roof.update({
        "kernel": (("ffn_stream_kernel / ffn_stream_bf16_kernel (the whole network in one launch)" if wl.C <= 64 else
                    "pointwise_kernel (first layer, GELU in its epilogue) + ffn_branch_kernel + pointwise_kernel (second layer)")
                   + ("; then forward_kernel (F_res) + pointwise_kernel (Conv_fuse, residual)" if ffn == "step" else "")
                   if ffn is not None else
                   f"forward_kernel<{wl.Ks}, RY, {'float' if wl.dtype == wk.F32 else 'bf16'}> (the only kernel of a step)"
                   if fused is None and not args.dense and not args.backward else
                   "corr_mfma_kernel (grad_out x correlation on the matrix cores), sums, estimator kernels, forward_kernel on grad_out with flipped kernels and the GAP term"
                   if args.backward else
                   "dense_bf16_kernel / dense_kernel (implicit GEMM on the matrix cores, DK taps, pass-through share) after the estimator launch and the weight rearrangement"
                   if args.dense else
                   "forward_kernel (F_res into the workspace) + pointwise_kernel (Conv_fuse on the matrix cores)"
                   + ("; with LK^c also the estimator launch and a second pointwise_kernel" if args.lkc else "")),
        "traffic": traffic, "traffic_source": traffic_src,
        # one step is one launch of the single forward kernel, so the per-launch duration is
        # the HIP-event time of a timed region divided by the number of launches in it
        "kernel_us": ms_step * 1e3,
    })
    res = {
        "metric": ("convffn_fwd_mpixel_per_s" if ffn == "ffn" else "esc_residual_step_fwd_mpixel_per_s" if ffn == "step" else
                   "convattn_dense_fwd_mpixel_per_s" if args.dense else "convattn_bwd_mpixel_per_s" if args.backward else
                   "convattn_fwd_mpixel_per_s" if fused is None else "convattn_fused_fwd_mpixel_per_s"),
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
        "config": {"workload": wl_name, "N": wl.N, "C": wl.C, "C_a": wl.Ca, "H": wl.H, "W": wl.W,
                   "Ks": wl.Ks, "launch": "eager" if args.eager else "hipgraph",
                   "buffer_pairs": max(2, int(-(-args.rotate_bytes // (2.0 * wl.N * wl.C * wl.H * wl.W * wl.elem_bytes))))
                   if not args.warm_cache else 1,
                   "cache": "warm" if args.warm_cache else "rotating", "replays": replays,
                   "statistic": "median over the replays of (replay time / steps)"},
        "ms_per_step_min": t["min"], "ms_per_step_max": t["max"], "ms_per_step_first_replay": t["first"],
        "single_call_latency_us": latency_us,
        "hbm_gbps_algorithmic": roof["hbm_gbps"],
        "valu_tflops": roof["alu_tflops"],
        "roofline": roof,
    }
    if floors is not None:
        res["floor"] = floors

    if not args.no_all_workloads:
        # every other benchmark workload, 200 launches per replay, no CPU leg
        others = []
        todo = [(i, None) for i in (0, 1, 2, 3)] + [(4, k) for k in wk.CFG4_KS] + [(5, None)]
        for idx, ks in todo:
            # (5: the larger model's shape, C = 192, C_a = 48, a hidden layer of 24)
            w2 = wk.make_large_model() if idx == 5 else wk.make_config(idx, ks) if idx == 4 else wk.make_config(idx)
            if w2.name == wl.name:
                continue
            r2 = Runner(w2, args.rotate_bytes, args.warm_cache)
            t2 = r2.time(200, 200, 25, eager=args.eager)
            s2 = t2["median"] * 1e-3
            rf = roofline_of(w2, s2)
            others.append({"workload": w2.name, "dtype": wk.DTYPE_NAMES[w2.dtype], "us_per_step": t2["median"] * 1e3,
                           "mpixel_per_s": w2.pixels / s2 / 1e6, "bound": rf["bound"], "frac": rf["frac"],
                           "hbm_gbps": rf["hbm_gbps"], "alu_tflops": rf["alu_tflops"],
                           "frac_of_roof_unpacked": rf["frac_of_roof_unpacked"],
                           "steps": 200, "warmup": 200, "replays": 25})
            del r2
            torch.cuda.empty_cache()
        res["all_workloads"] = others
        # the module with Conv_fuse (esc_convattn_fused_forward) on the benchmark shapes
        fus = []
        for idx, opts in ((1, {"lkc": False, "residual": False}), (1, {"lkc": True, "residual": True}),
                          (2, {"lkc": False, "residual": False}), (3, {"lkc": False, "residual": False})):
            w2 = wk.make_config(idx)
            name2 = w2.name + "_fused" + ("_lkc" if opts["lkc"] else "") + ("_res" if opts["residual"] else "")
            if fused is not None and name2 == wl_name:
                continue
            r2 = Runner(w2, args.rotate_bytes, args.warm_cache, fused=opts)
            t2 = r2.time(200, 200, 25, eager=args.eager)
            s2 = t2["median"] * 1e-3
            rf = fused_roofline_of(w2, s2, opts["lkc"], opts["residual"])
            fus.append({"workload": name2, "dtype": wk.DTYPE_NAMES[w2.dtype], "us_per_step": t2["median"] * 1e3,
                        "mpixel_per_s": w2.pixels / s2 / 1e6, "bound": rf["bound"], "frac": rf["frac"],
                        "hbm_gbps": rf["hbm_gbps"], "mfma_tflops": rf["mfma_tflops"], "alu_tflops": rf["alu_tflops"],
                        "steps": 200, "warmup": 200, "replays": 25})
            del r2
            torch.cuda.empty_cache()
        res["fused_workloads"] = fus
        # the module with the dense 13 x 13 x 16 x 16 large kernel of the paper's main variants
        den = []
        for idx in (1, 2):
            w2 = wk.make_config(idx)
            if args.dense and w2.name + "_dense" == wl_name:
                continue
            r2 = Runner(w2, args.rotate_bytes, args.warm_cache, dense=True)
            t2 = r2.time(100, 100, 15, eager=args.eager)
            s2 = t2["median"] * 1e-3
            rf = dense_roofline_of(w2, s2)
            den.append({"workload": w2.name + "_dense", "dtype": wk.DTYPE_NAMES[w2.dtype], "us_per_step": t2["median"] * 1e3,
                        "mpixel_per_s": w2.pixels / s2 / 1e6, "bound": rf["bound"], "frac": rf["frac"],
                        "hbm_gbps": rf["hbm_gbps"], "mfma_tflops": rf["mfma_tflops"], "steps": 100, "warmup": 100, "replays": 15})
            del r2
            torch.cuda.empty_cache()
        res["dense_workloads"] = den
        # the backward of the depth-wise module
        bwd = []
        for idx in (1, 3):
            w2 = wk.make_config(idx)
            if args.backward and w2.name + "_backward" == wl_name:
                continue
            r2 = Runner(w2, args.rotate_bytes, args.warm_cache, backward=True)
            t2 = r2.time(100, 100, 15, eager=args.eager)
            s2 = t2["median"] * 1e-3
            rf = backward_roofline_of(w2, s2)
            bwd.append({"workload": w2.name + "_backward", "dtype": wk.DTYPE_NAMES[w2.dtype], "us_per_step": t2["median"] * 1e3,
                        "mpixel_per_s": w2.pixels / s2 / 1e6, "bound": rf["bound"], "frac": rf["frac"],
                        "hbm_gbps": rf["hbm_gbps"], "alu_tflops": rf["alu_tflops"], "steps": 100, "warmup": 100, "replays": 15})
            del r2
            torch.cuda.empty_cache()
        res["backward_workloads"] = bwd
        # ConvFFN (hidden width 2 C) and the whole residual step of Eq. 3 line 3
        ffs = []
        for idx, kind in ((1, "ffn"), (2, "ffn"), (1, "step"), (2, "step")):
            w2 = wk.make_config(idx)
            name2 = w2.name + ("_convffn" if kind == "ffn" else "_residual_step")
            if name2 == wl_name:
                continue
            r2 = Runner(w2, args.rotate_bytes, args.warm_cache, ffn=kind,
                        fused={"lkc": False, "residual": False} if kind == "step" else None)
            t2 = r2.time(100, 100, 15, eager=args.eager)
            s2 = t2["median"] * 1e-3
            rf = ffn_roofline_of(w2, s2, kind == "step")
            ffs.append({"workload": name2, "dtype": wk.DTYPE_NAMES[w2.dtype], "us_per_step": t2["median"] * 1e3,
                        "mpixel_per_s": w2.pixels / s2 / 1e6, "bound": rf["bound"], "frac": rf["frac"],
                        "hbm_gbps": rf["hbm_gbps"], "mfma_tflops": rf["mfma_tflops"], "steps": 100, "warmup": 100, "replays": 15})
            del r2
            torch.cuda.empty_cache()
        res["ffn_workloads"] = ffs

    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
