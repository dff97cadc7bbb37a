"""Seeded synthetic inputs for the ConvAttn forward pass.

This module only draws random tensors and converts storage formats.  It holds
none of the method's arithmetic, so both the CPU oracle's tests and the HIP
path's tests/bench may import it without sharing any computation.

The five workloads stand in for the feature maps the ESC paper feeds its
ConvAttn module (Sec. 3 "Convolutional Attention Module", Eq. 4): the HD-output
latency protocol of Table 2 (a 1280x720 output at x2 / x4 gives 640x360 and
320x180 low-resolution maps with C = 64 channels, 16 of them in the attention
slice) and the training batch of 64 patches of 64x64 (implementation details,
"Classic SR").  No dataset image or trained weight is used.

Draw order per workload (one numpy Generator per seed): per-image sigma (only
workload 3), x, large kernel(s), generator weight.  Everything is drawn in
float32 and, for bf16 workloads, x is rounded to bfloat16 (nearest-even) and
handed out as raw uint16 bit patterns.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

F32 = 0
BF16 = 1

DTYPE_NAMES = {F32: "f32", BF16: "bf16"}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    rounded = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    rounded = np.where(nan, (u >> 16) | 0x0040, rounded)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


@dataclasses.dataclass
class Workload:
    """One ConvAttn call's inputs, all host numpy arrays.

    x        [N,C,H,W]   float32, or uint16 bfloat16 bits when dtype == BF16
    lk       [Ca,Ks,Ks]  float32 depthwise large kernel, one filter per channel
    w_down   [h,Ca] / None, b_down [h] / None   first generator layer (hidden > 0)
    w_up     [9*Ca, Ca or h], b_up [9*Ca] / None
    """
    name: str
    dtype: int
    N: int
    C: int
    H: int
    W: int
    Ca: int
    Ks: int
    hidden: int
    x: np.ndarray
    lk: np.ndarray
    w_up: np.ndarray
    b_up: Optional[np.ndarray] = None
    w_down: Optional[np.ndarray] = None
    b_down: Optional[np.ndarray] = None

    @property
    def pixels(self) -> int:
        return self.N * self.H * self.W

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2

    def x_as_f32(self) -> np.ndarray:
        return self.x if self.dtype == F32 else bf16_bits_to_f32(self.x)


# (N, C, Ca, H, W, dtype, seed, default Ks)
_CONFIGS = {
    0: ("cfg0_tiny_64x64_f32", 1, 64, 16, 64, 64, F32, 0),
    1: ("cfg1_hd_x4_180x320_f32", 1, 64, 16, 180, 320, F32, 1),
    2: ("cfg2_hd_x2_360x640_bf16", 1, 64, 16, 360, 640, BF16, 2),
    3: ("cfg3_train_batch_64x64x64_bf16", 64, 64, 16, 64, 64, BF16, 3),
    4: ("cfg4_1080p_x2_540x960_f32", 1, 64, 16, 540, 960, F32, 4),
}
CFG4_KS = (7, 13, 17, 31)


def config_shape(idx: int):
    name, N, C, Ca, H, W, dtype, seed = _CONFIGS[idx]
    return dict(name=name, N=N, C=C, Ca=Ca, H=H, W=W, dtype=dtype, seed=seed)


def make_config(idx: int, Ks: Optional[int] = None) -> Workload:
    """Build benchmark workload `idx` (0..4).  Workload 4 takes Ks in CFG4_KS."""
    name, N, C, Ca, H, W, dtype, seed = _CONFIGS[idx]
    rng = np.random.default_rng(seed)
    if idx == 3:
        sigma = rng.uniform(0.5, 2.0, size=N).astype(np.float32)
        x = rng.standard_normal((N, C, H, W), dtype=np.float32) * sigma[:, None, None, None]
    else:
        x = rng.standard_normal((N, C, H, W), dtype=np.float32)
    if idx == 4:
        if Ks is None:
            Ks = 13
        if Ks not in CFG4_KS:
            raise ValueError(f"workload 4 is defined for Ks in {CFG4_KS}")
        lk = None
        for k in CFG4_KS:  # kernels are drawn in this fixed order so every Ks sees the same x
            cand = rng.standard_normal((Ca, k, k), dtype=np.float32) * np.float32(1.0 / k)
            if k == Ks:
                lk = cand
        name = f"{name}_ks{Ks}"
    else:
        if Ks not in (None, 13):
            raise ValueError("workloads 0-3 are defined for Ks = 13")
        Ks = 13
        lk = rng.standard_normal((Ca, Ks, Ks), dtype=np.float32) * np.float32(1.0 / Ks)
    # drawn after every kernel so the generator weight does not depend on Ks
    w_up = rng.standard_normal((9 * Ca, Ca), dtype=np.float32) * np.float32(0.25)
    if dtype == BF16:
        x = f32_to_bf16_bits(x)
    return Workload(name=name, dtype=dtype, N=N, C=C, H=H, W=W, Ca=Ca, Ks=Ks, hidden=0,
                    x=np.ascontiguousarray(x), lk=np.ascontiguousarray(lk), w_up=w_up)


def make_large_model() -> Workload:
    """The ConvAttn call of the paper's scaled-up model (appendix "Classic SR Results on
    Larger Model Size": C = 192, 48 attention channels, two-layer estimator with h = 24) on
    the 320x180 map of the x4 HD protocol.  Not one of the five benchmark workloads: a
    second measured point for the two-layer estimator.  x_mean = 0.25 keeps DK visible."""
    wl = make_random(5, 1, 192, 180, 320, 48, 13, dtype=F32, hidden=24, bias=True, x_mean=0.25)
    wl.name = "large_model_c192_ca48_h24_180x320_f32"
    return wl


def make_random(seed: int, N: int, C: int, H: int, W: int, Ca: int, Ks: int, dtype: int = F32,
                hidden: int = 0, bias: bool = False, x_mean: float = 0.0,
                x_scale: float = 1.0) -> Workload:
    """Free-form seeded workload for unit and edge-case tests.

    hidden > 0 selects the paper's two-layer kernel estimator (1x1 down, GELU,
    1x1 up); hidden == 0 the single linear layer of the benchmark workloads.
    """
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((N, C, H, W), dtype=np.float32) * np.float32(x_scale)
         + np.float32(x_mean))
    lk = rng.standard_normal((Ca, Ks, Ks), dtype=np.float32) * np.float32(1.0 / Ks)
    w_down = b_down = b_up = None
    if hidden > 0:
        w_down = rng.standard_normal((hidden, max(Ca, 1)), dtype=np.float32)[:, :Ca] \
            * np.float32(1.0 / np.sqrt(max(Ca, 1)))
        w_down = np.ascontiguousarray(w_down)
        w_up = rng.standard_normal((9 * Ca, hidden), dtype=np.float32) * np.float32(1.0 / np.sqrt(hidden))
        if bias:
            b_down = rng.standard_normal(hidden, dtype=np.float32) * np.float32(0.1)
    else:
        w_up = rng.standard_normal((9 * Ca, max(Ca, 1)), dtype=np.float32)[:, :Ca] \
            * np.float32(1.0 / np.sqrt(max(Ca, 1)))
        w_up = np.ascontiguousarray(w_up)
    if bias:
        b_up = rng.standard_normal(9 * Ca, dtype=np.float32) * np.float32(0.1)
    if dtype == BF16:
        x = f32_to_bf16_bits(x)
    return Workload(name=f"rand_s{seed}_{N}x{C}x{H}x{W}_ca{Ca}_ks{Ks}_{DTYPE_NAMES[dtype]}_h{hidden}",
                    dtype=dtype, N=N, C=C, H=H, W=W, Ca=Ca, Ks=Ks, hidden=hidden,
                    x=np.ascontiguousarray(x), lk=np.ascontiguousarray(lk), w_up=w_up, b_up=b_up,
                    w_down=w_down, b_down=b_down)


def make_ffn_params(seed: int, C: int, Ch: int, bias: bool = True):
    """Seeded ConvFFN parameters (Eq. 3: the feed-forward network in front of the module):
    w1[Ch,C] ~ N(0,1/C), k[Ch,3,3] ~ N(0,1/9), w2[C,Ch] ~ N(0,1/Ch), biases ~ N(0,0.01)
    or None.  Returns a dict of float32 arrays."""
    rng = np.random.default_rng(seed)
    p = {
        "w1": rng.standard_normal((Ch, C), dtype=np.float32) * np.float32(1.0 / np.sqrt(C)),
        "k": rng.standard_normal((Ch, 3, 3), dtype=np.float32) * np.float32(1.0 / 3.0),
        "w2": rng.standard_normal((C, Ch), dtype=np.float32) * np.float32(1.0 / np.sqrt(Ch)),
        "b1": None, "bk": None, "b2": None,
    }
    if bias:
        p["b1"] = rng.standard_normal(Ch, dtype=np.float32) * np.float32(0.1)
        p["bk"] = rng.standard_normal(Ch, dtype=np.float32) * np.float32(0.1)
        p["b2"] = rng.standard_normal(C, dtype=np.float32) * np.float32(0.1)
    return p
