"""ctypes front end of the CPU oracle (oracle/esc_oracle.c).

TEST INFRASTRUCTURE ONLY: used by tests/, the smoke check and the benchmark's
cpu_baseline leg.  The product path never imports this module.

Each function mirrors one C entry point; see the C file for the passages of the
ESC paper (Sec. 3, Eq. 4 and the paragraph around Eq. 5) each one follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("esc_oracle.c", "esc_oracle_fuse.c", "esc_oracle_dense.c", "esc_oracle_backward.c",
                                            "esc_oracle_ffn.c")]
_LIB = os.path.join(_HERE, "libesc_oracle.so")

F32 = 0
BF16 = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (a second or two).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(s) for s in _SRCS):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", "-o", _LIB, *_SRCS, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ci, cl = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
        lib.esc_oracle_gap.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp]
        lib.esc_oracle_gap.restype = None
        lib.esc_oracle_generator.argtypes = [vp, ci, ci, ci, vp, vp, vp, vp, vp]
        lib.esc_oracle_generator.restype = None
        lib.esc_oracle_lk_conv.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci, cl, vp]
        lib.esc_oracle_lk_conv.restype = None
        lib.esc_oracle_dk_conv.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp]
        lib.esc_oracle_dk_conv.restype = None
        lib.esc_oracle_convattn_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci, cl,
                                                    ci, ci, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.esc_oracle_convattn_forward.restype = ci
        lib.esc_oracle_pointwise_lkc.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp]
        lib.esc_oracle_pointwise_lkc.restype = None
        lib.esc_oracle_fuse_1x1.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp]
        lib.esc_oracle_fuse_1x1.restype = None
        lib.esc_oracle_convattn_fused_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp, ci, cl,
                                                          ci, ci, vp, vp, vp, vp, vp, vp, vp, vp,
                                                          vp, vp, vp]
        lib.esc_oracle_convattn_fused_forward.restype = ci
        lib.esc_oracle_dense_lk_conv.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci, vp]
        lib.esc_oracle_dense_lk_conv.restype = None
        lib.esc_oracle_convattn_dense_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci, ci, ci,
                                                          vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.esc_oracle_convattn_dense_forward.restype = ci
        lib.esc_oracle_convattn_backward.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, ci, cl, ci, ci, vp, vp, vp, vp,
                                                     vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.esc_oracle_convattn_backward.restype = ci
        lib.esc_oracle_ffn_expand.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp, vp]
        lib.esc_oracle_ffn_expand.restype = None
        lib.esc_oracle_ffn_dwbranch.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp]
        lib.esc_oracle_ffn_dwbranch.restype = None
        lib.esc_oracle_ffn_project.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp, vp]
        lib.esc_oracle_ffn_project.restype = None
        lib.esc_oracle_convffn_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp]
        lib.esc_oracle_convffn_forward.restype = ci
        lib.esc_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        lib.esc_oracle_f32_to_bf16.restype = ctypes.c_uint16
        lib.esc_oracle_threads.restype = ci
        lib.esc_oracle_set_threads.argtypes = [ci]
        _lib = lib
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _x(x: np.ndarray, dtype: int) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16
    if x.dtype != want:
        raise TypeError(f"x must be {want} for dtype {dtype}")
    if x.ndim != 4:
        raise ValueError("x must be [N,C,H,W]")
    return np.ascontiguousarray(x)


def _f32(a: Optional[np.ndarray]) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def threads() -> int:
    return _load().esc_oracle_threads()


def set_threads(t: int) -> None:
    _load().esc_oracle_set_threads(int(t))


def f32_to_bf16(v: float) -> int:
    return int(_load().esc_oracle_f32_to_bf16(ctypes.c_float(v)))


def gap(x: np.ndarray, Ca: int, dtype: int = F32) -> np.ndarray:
    """Global average pool of the attention slice -> [N,Ca] float64."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    g = np.empty((N, Ca), dtype=np.float64)
    _load().esc_oracle_gap(_ptr(x), dtype, N, C, H, W, Ca, _ptr(g))
    return g


def generator(g: np.ndarray, hidden: int, w_up: np.ndarray, b_up=None, w_down=None,
              b_down=None) -> np.ndarray:
    """Kernel estimator -> DK [N,Ca,3,3] float64."""
    g = np.ascontiguousarray(g, dtype=np.float64)
    N, Ca = g.shape
    w_up, b_up, w_down, b_down = _f32(w_up), _f32(b_up), _f32(w_down), _f32(b_down)
    K = hidden if hidden > 0 else Ca
    assert w_up.shape == (9 * Ca, K), (w_up.shape, (9 * Ca, K))
    if hidden > 0:
        assert w_down.shape == (hidden, Ca)
    dk = np.empty((N, Ca, 3, 3), dtype=np.float64)
    _load().esc_oracle_generator(_ptr(g), N, Ca, hidden, _ptr(w_down), _ptr(b_down), _ptr(w_up),
                                 _ptr(b_up), _ptr(dk))
    return dk


def _lk_stride(lk: np.ndarray, Ca: int):
    lk = _f32(lk)
    if lk.ndim == 2:
        return lk, lk.shape[0], 0
    assert lk.ndim == 3 and lk.shape[0] == Ca and lk.shape[1] == lk.shape[2]
    return lk, lk.shape[1], lk.shape[1] * lk.shape[2]


def lk_conv(x: np.ndarray, Ca: int, lk: np.ndarray, dtype: int = F32) -> np.ndarray:
    """F_att cross-correlated with the large kernel -> [N,Ca,H,W] float64."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    lk, Ks, cs = _lk_stride(lk, Ca)
    res = np.empty((N, Ca, H, W), dtype=np.float64)
    _load().esc_oracle_lk_conv(_ptr(x), dtype, N, C, H, W, Ca, _ptr(lk), Ks, cs, _ptr(res))
    return res


def dk_conv(x: np.ndarray, Ca: int, dk: np.ndarray, dtype: int = F32) -> np.ndarray:
    """F_att cross-correlated with a per-image 3x3 kernel -> [N,Ca,H,W] float64."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    dk = np.ascontiguousarray(dk, dtype=np.float64)
    assert dk.shape == (N, Ca, 3, 3)
    res = np.empty((N, Ca, H, W), dtype=np.float64)
    _load().esc_oracle_dk_conv(_ptr(x), dtype, N, C, H, W, Ca, _ptr(dk), _ptr(res))
    return res


def convattn_forward(x: np.ndarray, Ca: int, lk: np.ndarray, dtype: int = F32, *,
                     hidden: int = 0, w_up=None, b_up=None, w_down=None, b_down=None,
                     dk_in=None, want_out: bool = True):
    """Whole forward.  DK comes from the estimator when w_up is given, from
    dk_in when that is given, and is zero when neither is.

    Returns (res_att float64 [N,Ca,H,W], dk float64 [N,Ca,3,3], out in storage
    dtype [N,C,H,W] or None).
    """
    x = _x(x, dtype)
    N, C, H, W = x.shape
    lk, Ks, cs = _lk_stride(lk, Ca)
    if w_up is not None and dk_in is not None:
        raise ValueError("give either estimator weights or dk_in, not both")
    mode = 1 if w_up is not None else (2 if dk_in is not None else 0)
    w_up, b_up, w_down, b_down = _f32(w_up), _f32(b_up), _f32(w_down), _f32(b_down)
    if mode == 1:
        K = hidden if hidden > 0 else Ca
        assert w_up.shape == (9 * Ca, K)
        if hidden > 0:
            assert w_down.shape == (hidden, Ca)
    if dk_in is not None:
        dk_in = np.ascontiguousarray(dk_in, dtype=np.float64)
        assert dk_in.shape == (N, Ca, 3, 3)
    res = np.empty((N, Ca, H, W), dtype=np.float64)
    dk = np.empty((N, Ca, 3, 3), dtype=np.float64)
    out = np.empty_like(x) if want_out else None
    rc = _load().esc_oracle_convattn_forward(
        _ptr(x), dtype, N, C, H, W, Ca, _ptr(lk), Ks, cs, mode, hidden,
        _ptr(w_down), _ptr(b_down), _ptr(w_up), _ptr(b_up), _ptr(dk_in),
        _ptr(res), _ptr(dk), _ptr(out))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return res, dk, out


def forward_workload(wl, want_out: bool = True):
    """Run the whole forward on a workloads.Workload-like object."""
    return convattn_forward(wl.x, wl.Ca, wl.lk, wl.dtype, hidden=wl.hidden, w_up=wl.w_up,
                            b_up=wl.b_up, w_down=wl.w_down, b_down=wl.b_down, want_out=want_out)


# ---------------------------------------------------------------- point-wise steps (esc_oracle_fuse.c)

def pointwise_lkc(x: np.ndarray, Ca: int, lkc: np.ndarray, dtype: int = F32) -> np.ndarray:
    """F_att (*) LK^c, the first factor of Eq. 5 -> [N,Ca,H,W] float64."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    lkc = _f32(lkc)
    assert lkc.shape == (Ca, Ca)
    pw = np.empty((N, Ca, H, W), dtype=np.float64)
    _load().esc_oracle_pointwise_lkc(_ptr(x), dtype, N, C, H, W, Ca, _ptr(lkc), _ptr(pw))
    return pw


def fuse_1x1(cat: np.ndarray, w: np.ndarray, b=None) -> np.ndarray:
    """Conv_fuse 1x1 (Eq. 4 line 4) of a float64 [N,C,H,W] tensor -> float64 [N,C,H,W]."""
    cat = np.ascontiguousarray(cat, dtype=np.float64)
    N, C, H, W = cat.shape
    w, b = _f32(w), _f32(b)
    assert w.shape == (C, C) and (b is None or b.shape == (C,))
    out = np.empty_like(cat)
    _load().esc_oracle_fuse_1x1(_ptr(cat), N, C, H, W, _ptr(w), _ptr(b), _ptr(out))
    return out


def convattn_fused_forward(x: np.ndarray, Ca: int, lk: np.ndarray, w_fuse: np.ndarray, dtype: int = F32, *,
                           b_fuse=None, lkc=None, residual=None, hidden: int = 0, w_up=None, b_up=None,
                           w_down=None, b_down=None, dk_in=None):
    """The module with Conv_fuse, optionally LK^c in front (Eq. 5) and the residual of Eq. 3.

    Returns (out float64 [N,C,H,W], res_att float64 [N,Ca,H,W], dk float64 [N,Ca,3,3]).
    """
    x = _x(x, dtype)
    N, C, H, W = x.shape
    lk, Ks, cs = _lk_stride(lk, Ca)
    if w_up is not None and dk_in is not None:
        raise ValueError("give either estimator weights or dk_in, not both")
    mode = 1 if w_up is not None else (2 if dk_in is not None else 0)
    w_up, b_up, w_down, b_down = _f32(w_up), _f32(b_up), _f32(w_down), _f32(b_down)
    w_fuse, b_fuse, lkc = _f32(w_fuse), _f32(b_fuse), _f32(lkc)
    assert w_fuse.shape == (C, C) and (b_fuse is None or b_fuse.shape == (C,))
    assert lkc is None or lkc.shape == (Ca, Ca)
    if mode == 1:
        K = hidden if hidden > 0 else Ca
        assert w_up.shape == (9 * Ca, K)
        if hidden > 0:
            assert w_down.shape == (hidden, Ca)
    if dk_in is not None:
        dk_in = np.ascontiguousarray(dk_in, dtype=np.float64)
        assert dk_in.shape == (N, Ca, 3, 3)
    if residual is not None:
        residual = _x(residual, dtype)
        assert residual.shape == x.shape
    res = np.empty((N, Ca, H, W), dtype=np.float64)
    dk = np.empty((N, Ca, 3, 3), dtype=np.float64)
    out = np.empty((N, C, H, W), dtype=np.float64)
    rc = _load().esc_oracle_convattn_fused_forward(
        _ptr(x), dtype, N, C, H, W, Ca, _ptr(lkc), _ptr(lk), Ks, cs, mode, hidden,
        _ptr(w_down), _ptr(b_down), _ptr(w_up), _ptr(b_up), _ptr(dk_in), _ptr(w_fuse), _ptr(b_fuse),
        _ptr(residual), _ptr(res), _ptr(dk), _ptr(out))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out, res, dk


# ---------------------------------------------------------------- dense large kernel (esc_oracle_dense.c)

def dense_lk_conv(x: np.ndarray, Ca: int, lk: np.ndarray, dtype: int = F32) -> np.ndarray:
    """F_att cross-correlated with a dense large kernel lk[Ca(out),Ca(in),Ks,Ks] -> [N,Ca,H,W] float64."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    lk = _f32(lk)
    assert lk.ndim == 4 and lk.shape[0] == lk.shape[1] == Ca and lk.shape[2] == lk.shape[3]
    res = np.empty((N, Ca, H, W), dtype=np.float64)
    _load().esc_oracle_dense_lk_conv(_ptr(x), dtype, N, C, H, W, Ca, _ptr(lk), lk.shape[2], _ptr(res))
    return res


def convattn_dense_forward(x: np.ndarray, Ca: int, lk: np.ndarray, dtype: int = F32, *, hidden: int = 0,
                           w_up=None, b_up=None, w_down=None, b_down=None, dk_in=None, want_out: bool = True):
    """The module with the dense large kernel of the paper's main variants (Eq. 4 lines 1-4
    without Conv_fuse).  Returns (res_att float64, dk float64, out in the storage dtype or None)."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    lk = _f32(lk)
    assert lk.ndim == 4 and lk.shape[0] == lk.shape[1] == Ca and lk.shape[2] == lk.shape[3]
    if w_up is not None and dk_in is not None:
        raise ValueError("give either estimator weights or dk_in, not both")
    mode = 1 if w_up is not None else (2 if dk_in is not None else 0)
    w_up, b_up, w_down, b_down = _f32(w_up), _f32(b_up), _f32(w_down), _f32(b_down)
    if mode == 1:
        K = hidden if hidden > 0 else Ca
        assert w_up.shape == (9 * Ca, K)
        if hidden > 0:
            assert w_down.shape == (hidden, Ca)
    if dk_in is not None:
        dk_in = np.ascontiguousarray(dk_in, dtype=np.float64)
        assert dk_in.shape == (N, Ca, 3, 3)
    res = np.empty((N, Ca, H, W), dtype=np.float64)
    tmp = np.empty((N, Ca, H, W), dtype=np.float64)
    dk = np.empty((N, Ca, 3, 3), dtype=np.float64)
    out = np.empty_like(x) if want_out else None
    rc = _load().esc_oracle_convattn_dense_forward(
        _ptr(x), dtype, N, C, H, W, Ca, _ptr(lk), lk.shape[2], mode, hidden, _ptr(w_down), _ptr(b_down),
        _ptr(w_up), _ptr(b_up), _ptr(dk_in), _ptr(tmp), _ptr(res), _ptr(dk), _ptr(out))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return res, dk, out


# ---------------------------------------------------------------- backward (esc_oracle_backward.c)

def convattn_backward(x: np.ndarray, go: np.ndarray, Ca: int, lk: np.ndarray, dtype: int = F32, *, hidden: int = 0,
                      w_up=None, b_up=None, w_down=None, b_down=None, dk_in=None):
    """Gradients of the depth-wise ConvAttn forward (Eq. 4 lines 1-4 without Conv_fuse) for an upstream
    gradient go = dL/dout.  Returns a dict of float64 arrays: dx [N,C,H,W], dlk (shape of lk), ddk [N,Ca,3,3],
    dg [N,Ca] and, when estimator weights are given, dw_up, db_up (and dw_down, db_down when hidden > 0)."""
    x, go = _x(x, dtype), _x(go, dtype)
    assert go.shape == x.shape
    N, C, H, W = x.shape
    lk, Ks, cs = _lk_stride(lk, Ca)
    if w_up is not None and dk_in is not None:
        raise ValueError("give either estimator weights or dk_in, not both")
    mode = 1 if w_up is not None else (2 if dk_in is not None else 0)
    w_up, b_up, w_down, b_down = _f32(w_up), _f32(b_up), _f32(w_down), _f32(b_down)
    K = hidden if hidden > 0 else Ca
    if mode == 1:
        assert w_up.shape == (9 * Ca, K)
        if hidden > 0:
            assert w_down.shape == (hidden, Ca)
    if dk_in is not None:
        dk_in = np.ascontiguousarray(dk_in, dtype=np.float64)
        assert dk_in.shape == (N, Ca, 3, 3)
    res = {"dx": np.empty((N, C, H, W)), "dlk": np.empty(lk.shape), "ddk": np.empty((N, Ca, 3, 3)),
           "dg": np.empty((N, Ca))}
    if mode == 1:
        res["dw_up"], res["db_up"] = np.empty((9 * Ca, K)), np.empty(9 * Ca)
        if hidden > 0:
            res["dw_down"], res["db_down"] = np.empty((hidden, Ca)), np.empty(hidden)
    rc = _load().esc_oracle_convattn_backward(
        _ptr(x), _ptr(go), dtype, N, C, H, W, Ca, _ptr(lk), Ks, cs, mode, hidden, _ptr(w_down), _ptr(b_down),
        _ptr(w_up), _ptr(b_up), _ptr(dk_in), _ptr(res["dx"]), _ptr(res["dlk"]), _ptr(res["ddk"]),
        _ptr(res.get("dw_up")), _ptr(res.get("db_up")), _ptr(res.get("dw_down")), _ptr(res.get("db_down")),
        _ptr(res["dg"]))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return res


# ---------------------------------------------------------------- ConvFFN (esc_oracle_ffn.c)

def ffn_expand(x: np.ndarray, w1: np.ndarray, b1=None, dtype: int = F32) -> np.ndarray:
    """First point-wise layer with its GELU -> [N,Ch,H,W] float64."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    w1, b1 = _f32(w1), _f32(b1)
    Ch = w1.shape[0]
    assert w1.shape == (Ch, C) and (b1 is None or b1.shape == (Ch,))
    u = np.empty((N, Ch, H, W), dtype=np.float64)
    _load().esc_oracle_ffn_expand(_ptr(x), dtype, N, C, H, W, Ch, _ptr(w1), _ptr(b1), _ptr(u))
    return u


def ffn_dwbranch(u: np.ndarray, k: np.ndarray, bk=None) -> np.ndarray:
    """u + gelu(depth-wise 3x3 of u) on a float64 [N,Ch,H,W] tensor -> float64."""
    u = np.ascontiguousarray(u, dtype=np.float64)
    N, Ch, H, W = u.shape
    k, bk = _f32(k), _f32(bk)
    assert k.shape == (Ch, 3, 3) and (bk is None or bk.shape == (Ch,))
    v = np.empty_like(u)
    _load().esc_oracle_ffn_dwbranch(_ptr(u), N, Ch, H, W, _ptr(k), _ptr(bk), _ptr(v))
    return v


def ffn_project(v: np.ndarray, w2: np.ndarray, b2=None) -> np.ndarray:
    """Second point-wise layer on a float64 [N,Ch,H,W] tensor -> float64 [N,C,H,W]."""
    v = np.ascontiguousarray(v, dtype=np.float64)
    N, Ch, H, W = v.shape
    w2, b2 = _f32(w2), _f32(b2)
    C = w2.shape[0]
    assert w2.shape == (C, Ch) and (b2 is None or b2.shape == (C,))
    y = np.empty((N, C, H, W), dtype=np.float64)
    _load().esc_oracle_ffn_project(_ptr(v), N, C, H, W, Ch, _ptr(w2), _ptr(b2), _ptr(y))
    return y


def convffn_forward(x: np.ndarray, w1, k, w2, dtype: int = F32, *, b1=None, bk=None, b2=None) -> np.ndarray:
    """ConvFFN of Eq. 3 (two point-wise layers around a depth-wise 3x3 branch) -> float64 [N,C,H,W]."""
    x = _x(x, dtype)
    N, C, H, W = x.shape
    w1, b1, k, bk, w2, b2 = _f32(w1), _f32(b1), _f32(k), _f32(bk), _f32(w2), _f32(b2)
    Ch = w1.shape[0]
    assert w1.shape == (Ch, C) and k.shape == (Ch, 3, 3) and w2.shape == (C, Ch)
    assert (b1 is None or b1.shape == (Ch,)) and (bk is None or bk.shape == (Ch,)) and (b2 is None or b2.shape == (C,))
    out = np.empty((N, C, H, W), dtype=np.float64)
    rc = _load().esc_oracle_convffn_forward(_ptr(x), dtype, N, C, H, W, Ch, _ptr(w1), _ptr(b1), _ptr(k), _ptr(bk),
                                            _ptr(w2), _ptr(b2), _ptr(out))
    if rc != 0:
        raise ValueError("oracle rejected the arguments")
    return out
