"""Thin ctypes binding over libesc_convattn.so (include/esc_convattn.h).

Argument marshalling only: every step of the ConvAttn forward (Eq. 4 of the ESC
paper) runs in the HIP kernels.  torch supplies device memory and streams.
There is no CPU fallback; a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libesc_convattn.so")

ESC_F32 = 0
ESC_BF16 = 1

EXPORTS = ("esc_workspace_bytes", "esc_workspace_init", "esc_workspace_errors", "esc_dynkernel_gen",
           "esc_convattn_forward", "esc_convattn_forward_noalloc", "esc_fused_workspace_bytes",
           "esc_convattn_fused_forward", "esc_dense_workspace_bytes", "esc_convattn_dense_forward",
           "esc_backward_workspace_bytes", "esc_convattn_backward", "esc_convffn_workspace_bytes",
           "esc_convffn_forward", "esc_residual_step_workspace_bytes", "esc_residual_step_forward", "esc_status_string")
NOALLOC_SCRATCH_BYTES = 1 << 20


class EscError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"esc_convattn: status {status}: {message}")
        self.status = status


class _GenParams(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int),
                ("w_down", ctypes.c_void_p), ("b_down", ctypes.c_void_p),
                ("w_up", ctypes.c_void_p), ("b_up", ctypes.c_void_p)]


class _GenGrads(ctypes.Structure):
    _fields_ = [("w_down", ctypes.c_void_p), ("b_down", ctypes.c_void_p),
                ("w_up", ctypes.c_void_p), ("b_up", ctypes.c_void_p)]


_lib = None


def load_library():
    """Load the built library; raise (never fall back) when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2503_06671_amd.build` "
                "(or __graft_entry__.build()) first")
        lib = ctypes.CDLL(LIB_PATH)
        vp, ci, cl, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_long, ctypes.c_size_t
        lib.esc_workspace_bytes.argtypes = [ci, ci, ci, ci]
        lib.esc_workspace_bytes.restype = sz
        lib.esc_workspace_init.argtypes = [vp, sz, vp]
        lib.esc_workspace_init.restype = ci
        lib.esc_workspace_errors.argtypes = [vp, sz, vp, ctypes.POINTER(ctypes.c_uint)]
        lib.esc_workspace_errors.restype = ci
        lib.esc_dynkernel_gen.argtypes = [vp, ci, ci, ci, ci, ci, ci, ctypes.POINTER(_GenParams), vp,
                                          vp, sz, vp]
        lib.esc_dynkernel_gen.restype = ci
        lib.esc_convattn_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci, cl,
                                             ctypes.POINTER(_GenParams), vp, vp, vp, sz, vp]
        lib.esc_convattn_forward.restype = ci
        lib.esc_convattn_forward_noalloc.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci, cl,
                                                     ctypes.POINTER(_GenParams), vp, vp, vp]
        lib.esc_convattn_forward_noalloc.restype = ci
        lib.esc_fused_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
        lib.esc_fused_workspace_bytes.restype = sz
        lib.esc_convattn_fused_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp, ci, cl,
                                                   ctypes.POINTER(_GenParams), vp, vp, vp, vp, vp, vp, sz, vp]
        lib.esc_convattn_fused_forward.restype = ci
        lib.esc_dense_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        lib.esc_dense_workspace_bytes.restype = sz
        lib.esc_convattn_dense_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, ci,
                                                   ctypes.POINTER(_GenParams), vp, vp, vp, sz, vp]
        lib.esc_convattn_dense_forward.restype = ci
        lib.esc_backward_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
        lib.esc_backward_workspace_bytes.restype = sz
        lib.esc_convattn_backward.argtypes = [vp, vp, ci, ci, ci, ci, ci, ci, vp, ci, cl, ctypes.POINTER(_GenParams), vp,
                                              vp, vp, ctypes.POINTER(_GenGrads), vp, ci, vp, sz, vp]
        lib.esc_convattn_backward.restype = ci
        lib.esc_convffn_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        lib.esc_convffn_workspace_bytes.restype = sz
        lib.esc_convffn_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.esc_convffn_forward.restype = ci
        lib.esc_residual_step_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci, ci, ci]
        lib.esc_residual_step_workspace_bytes.restype = sz
        lib.esc_residual_step_forward.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, vp, vp, vp, ci, vp, vp, ci, cl,
                                                  ctypes.POINTER(_GenParams), vp, vp, vp, vp, sz, vp]
        lib.esc_residual_step_forward.restype = ci
        lib.esc_status_string.argtypes = [ci]
        lib.esc_status_string.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load_library().esc_status_string(int(status)).decode()


def _check(status: int) -> None:
    if status != 0:
        raise EscError(status, status_string(status))


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _dtype_of(x: torch.Tensor) -> int:
    if x.dtype == torch.float32:
        return ESC_F32
    if x.dtype == torch.bfloat16:
        return ESC_BF16
    raise TypeError(f"x must be float32 or bfloat16, got {x.dtype}")


def _dev_f32(t: Optional[torch.Tensor], name: str) -> Optional[torch.Tensor]:
    if t is None:
        return None
    if not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous():
        raise TypeError(f"{name} must be a contiguous float32 device tensor")
    return t


class GenParams:
    """Device weights of the kernel estimator (Eq. 4 line 2); see esc_gen_params."""

    def __init__(self, w_up: torch.Tensor, b_up: Optional[torch.Tensor] = None, hidden: int = 0,
                 w_down: Optional[torch.Tensor] = None, b_down: Optional[torch.Tensor] = None):
        self.tensors = (_dev_f32(w_down, "w_down"), _dev_f32(b_down, "b_down"),
                        _dev_f32(w_up, "w_up"), _dev_f32(b_up, "b_up"))
        self.hidden = int(hidden)
        self.c = _GenParams(self.hidden, *[_ptr(t) for t in self.tensors])

    def check(self, Ca: int) -> None:
        """The library reads these buffers by the sizes C_a and hidden imply: refuse others."""
        w_down, b_down, w_up, b_up = self.tensors
        K = self.hidden if self.hidden > 0 else Ca
        want = {"w_up": (w_up, 9 * Ca * K), "b_up": (b_up, 9 * Ca)}
        if self.hidden > 0:
            want["w_down"] = (w_down, self.hidden * Ca)
            want["b_down"] = (b_down, self.hidden)
            if w_down is None:
                raise ValueError("hidden > 0 needs w_down")
        for name, (tensor, numel) in want.items():
            if tensor is not None and tensor.numel() != numel:
                raise ValueError(f"{name} has {tensor.numel()} elements, C_a = {Ca} and hidden = {self.hidden} "
                                 f"need {numel}")


def workspace_bytes(N: int, Ca: int, H: int, W: int) -> int:
    return int(load_library().esc_workspace_bytes(N, Ca, H, W))


def workspace_init(ws: torch.Tensor, stream=None) -> None:
    _check(load_library().esc_workspace_init(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream)))


def workspace_errors(ws: torch.Tensor, stream=None) -> int:
    """Diagnostic: synchronises the stream and returns the workspace's error word."""
    v = ctypes.c_uint(0)
    _check(load_library().esc_workspace_errors(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream),
                                               ctypes.byref(v)))
    return int(v.value)


def new_workspace(N: int, Ca: int, H: int, W: int, device="cuda", stream=None) -> torch.Tensor:
    """Allocate (with torch) and prepare a workspace for this shape."""
    nbytes = workspace_bytes(N, Ca, H, W)
    if nbytes == 0:
        raise ValueError("bad shape for a workspace")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def _x_checked(x: torch.Tensor):
    if not x.is_cuda or x.dim() != 4 or not x.is_contiguous():
        raise TypeError("x must be a contiguous [N,C,H,W] device tensor")
    return _dtype_of(x), tuple(int(v) for v in x.shape)


def dynkernel_gen(x: torch.Tensor, Ca: int, gen: GenParams, workspace: torch.Tensor,
                  dk_out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """esc_dynkernel_gen: DK [N,Ca,3,3] float32 from GAP of the attention slice."""
    dt, (N, C, H, W) = _x_checked(x)
    gen.check(int(Ca))
    if dk_out is None:
        dk_out = torch.empty((N, Ca, 3, 3), dtype=torch.float32, device=x.device)
    _dev_f32(dk_out, "dk_out")
    if dk_out.numel() != N * Ca * 9:
        raise ValueError("dk_out must hold [N, Ca, 3, 3] values")
    _check(load_library().esc_dynkernel_gen(
        _ptr(x), dt, N, C, H, W, int(Ca), ctypes.byref(gen.c), _ptr(dk_out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
    return dk_out


def _lk_checked(lk: torch.Tensor, Ca: int, ks: Optional[int], lk_channel_stride: Optional[int]):
    """(Ks, channel stride) of the large kernel: [Ca,Ks,Ks] (one filter per channel), [Ks,Ks]
    (one for all), or a flat buffer read with an explicit Ks and channel stride."""
    _dev_f32(lk, "lk")
    if ks is not None or lk_channel_stride is not None:
        if ks is None or lk_channel_stride is None:
            raise ValueError("give ks and lk_channel_stride together")
        ks, stride = int(ks), int(lk_channel_stride)
        need = (Ca - 1) * stride + ks * ks if (stride and Ca > 0) else ks * ks
        if lk.numel() < need:
            raise ValueError(f"lk holds {lk.numel()} values, Ks = {ks} with channel stride {stride} reads {need}")
        return ks, stride
    if lk.dim() == 2 and lk.shape[0] == lk.shape[1]:
        return int(lk.shape[0]), 0
    if lk.dim() == 3 and lk.shape[1] == lk.shape[2] and (lk.shape[0] == Ca or Ca == 0):
        return int(lk.shape[1]), int(lk.shape[1] * lk.shape[2])
    raise ValueError(f"lk must be [Ca,Ks,Ks] with Ca = {Ca}, or [Ks,Ks]; got {tuple(lk.shape)}")


def convattn_forward(x: torch.Tensor, Ca: int, lk: torch.Tensor, workspace: Optional[torch.Tensor],
                     gen: Optional[GenParams] = None, dk_in: Optional[torch.Tensor] = None,
                     out: Optional[torch.Tensor] = None, stream=None, ks: Optional[int] = None,
                     lk_channel_stride: Optional[int] = None) -> torch.Tensor:
    """esc_convattn_forward (workspace given) or esc_convattn_forward_noalloc (workspace None).
    lk is [Ca,Ks,Ks] (one filter per channel) or [Ks,Ks] (shared); with ks and
    lk_channel_stride given it is a flat buffer with channel c at c * stride."""
    dt, (N, C, H, W) = _x_checked(x)
    Ks, stride = _lk_checked(lk, int(Ca), ks, lk_channel_stride)
    if gen is not None:
        gen.check(int(Ca))
    if out is None:
        out = torch.empty_like(x)
    if out.dtype != x.dtype or out.shape != x.shape or not out.is_contiguous():
        raise TypeError("out must match x in dtype and shape and be contiguous")
    _dev_f32(dk_in, "dk_in")
    if dk_in is not None and dk_in.numel() != N * Ca * 9:
        raise ValueError("dk_in must hold [N, Ca, 3, 3] values")
    gen_ref = ctypes.byref(gen.c) if gen is not None else None
    if workspace is None:  # the entry point that allocates nothing: the library's own scratch
        _check(load_library().esc_convattn_forward_noalloc(
            _ptr(x), dt, N, C, H, W, int(Ca), _ptr(lk), Ks, stride, gen_ref, _ptr(dk_in), _ptr(out),
            _stream(stream)))
        return out
    ws_ptr, ws_bytes = _ptr(workspace), workspace.numel() * workspace.element_size()
    _check(load_library().esc_convattn_forward(
        _ptr(x), dt, N, C, H, W, int(Ca), _ptr(lk), Ks, stride, gen_ref, _ptr(dk_in), _ptr(out),
        ws_ptr, ws_bytes, _stream(stream)))
    return out


def fused_workspace_bytes(N: int, Ca: int, H: int, W: int, dtype: torch.dtype, with_lk_c: bool) -> int:
    dt = ESC_F32 if dtype == torch.float32 else ESC_BF16
    return int(load_library().esc_fused_workspace_bytes(N, Ca, H, W, dt, int(bool(with_lk_c))))


def new_fused_workspace(N: int, Ca: int, H: int, W: int, dtype: torch.dtype, with_lk_c: bool, device="cuda",
                        stream=None) -> torch.Tensor:
    """Allocate (with torch) and prepare a workspace for esc_convattn_fused_forward."""
    nbytes = fused_workspace_bytes(N, Ca, H, W, dtype, with_lk_c)
    if nbytes == 0:
        raise ValueError("bad shape for a workspace")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def convattn_fused_forward(x: torch.Tensor, Ca: int, lk: torch.Tensor, w_fuse: torch.Tensor, workspace: torch.Tensor,
                           b_fuse: Optional[torch.Tensor] = None, lk_c: Optional[torch.Tensor] = None,
                           residual: Optional[torch.Tensor] = None, gen: Optional[GenParams] = None,
                           dk_in: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                           stream=None) -> torch.Tensor:
    """esc_convattn_fused_forward: the module with Conv_fuse, optionally LK^c and the residual."""
    dt, (N, C, H, W) = _x_checked(x)
    Ks, stride = _lk_checked(lk, int(Ca), None, None)
    if gen is not None:
        gen.check(int(Ca))
    _dev_f32(w_fuse, "w_fuse"), _dev_f32(b_fuse, "b_fuse"), _dev_f32(lk_c, "lk_c"), _dev_f32(dk_in, "dk_in")
    if w_fuse.numel() != C * C or (b_fuse is not None and b_fuse.numel() != C):
        raise ValueError("w_fuse must be [C, C] and b_fuse [C]")
    if lk_c is not None and lk_c.numel() != Ca * Ca:
        raise ValueError("lk_c must be [Ca, Ca]")
    if dk_in is not None and dk_in.numel() != N * Ca * 9:
        raise ValueError("dk_in must hold [N, Ca, 3, 3] values")
    if residual is not None and (residual.dtype != x.dtype or residual.shape != x.shape or not residual.is_contiguous()
                                 or not residual.is_cuda):
        raise TypeError("residual must match x in dtype and shape and be a contiguous device tensor")
    if out is None:
        out = torch.empty_like(x)
    if out.dtype != x.dtype or out.shape != x.shape or not out.is_contiguous():
        raise TypeError("out must match x in dtype and shape and be contiguous")
    _check(load_library().esc_convattn_fused_forward(
        _ptr(x), dt, N, C, H, W, int(Ca), _ptr(lk_c), _ptr(lk), Ks, stride,
        ctypes.byref(gen.c) if gen is not None else None, _ptr(dk_in), _ptr(w_fuse), _ptr(b_fuse), _ptr(residual),
        _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def new_convffn_workspace(N: int, Ch: int, H: int, W: int, dtype: torch.dtype, device="cuda") -> torch.Tensor:
    """Allocate (with torch) the scratch workspace of esc_convffn_forward (needs no preparation)."""
    dt = ESC_F32 if dtype == torch.float32 else ESC_BF16
    nbytes = int(load_library().esc_convffn_workspace_bytes(N, Ch, H, W, dt))
    if nbytes == 0:
        raise ValueError("bad shape for a workspace")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def convffn_forward(x: torch.Tensor, w1: torch.Tensor, k_dw: torch.Tensor, w2: torch.Tensor, workspace: torch.Tensor,
                    b1: Optional[torch.Tensor] = None, b_dw: Optional[torch.Tensor] = None,
                    b2: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """esc_convffn_forward: w1 [Ch, C], k_dw [Ch, 3, 3], w2 [C, Ch], optional biases."""
    dt, (N, C, H, W) = _x_checked(x)
    for t, name in ((w1, "w1"), (k_dw, "k_dw"), (w2, "w2"), (b1, "b1"), (b_dw, "b_dw"), (b2, "b2")):
        _dev_f32(t, name)
    if w1.dim() != 2 or w1.shape[1] != C:
        raise ValueError(f"w1 must be [Ch, C] with C = {C}; got {tuple(w1.shape)}")
    Ch = int(w1.shape[0])
    if tuple(k_dw.shape) != (Ch, 3, 3) or tuple(w2.shape) != (C, Ch):
        raise ValueError("k_dw must be [Ch, 3, 3] and w2 [C, Ch]")
    if (b1 is not None and b1.numel() != Ch) or (b_dw is not None and b_dw.numel() != Ch) or \
            (b2 is not None and b2.numel() != C):
        raise ValueError("b1 and b_dw must hold Ch values, b2 C values")
    if out is None:
        out = torch.empty_like(x)
    if out.dtype != x.dtype or out.shape != x.shape or not out.is_contiguous():
        raise TypeError("out must match x in dtype and shape and be contiguous")
    _check(load_library().esc_convffn_forward(
        _ptr(x), dt, N, C, H, W, Ch, _ptr(w1), _ptr(b1), _ptr(k_dw), _ptr(b_dw), _ptr(w2), _ptr(b2), _ptr(out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def new_residual_step_workspace(N: int, C: int, H: int, W: int, Ca: int, Ch: int, dtype: torch.dtype, with_lk_c: bool,
                                device="cuda", stream=None) -> torch.Tensor:
    """Allocate (with torch) and prepare a workspace for esc_residual_step_forward."""
    dt = ESC_F32 if dtype == torch.float32 else ESC_BF16
    nbytes = int(load_library().esc_residual_step_workspace_bytes(N, C, H, W, Ca, Ch, dt, int(bool(with_lk_c))))
    if nbytes == 0:
        raise ValueError("bad shape for a workspace")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def residual_step_forward(f_in: torch.Tensor, w1: torch.Tensor, k_dw: torch.Tensor, w2: torch.Tensor, Ca: int,
                          lk: torch.Tensor, w_fuse: torch.Tensor, workspace: torch.Tensor,
                          b1: Optional[torch.Tensor] = None, b_dw: Optional[torch.Tensor] = None,
                          b2: Optional[torch.Tensor] = None, lk_c: Optional[torch.Tensor] = None,
                          gen: Optional[GenParams] = None, b_fuse: Optional[torch.Tensor] = None,
                          out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """esc_residual_step_forward: f_in + ConvAttn(ConvFFN(f_in), LK) (Eq. 3 line 3)."""
    dt, (N, C, H, W) = _x_checked(f_in)
    for t, name in ((w1, "w1"), (k_dw, "k_dw"), (w2, "w2"), (b1, "b1"), (b_dw, "b_dw"), (b2, "b2"),
                    (w_fuse, "w_fuse"), (b_fuse, "b_fuse"), (lk_c, "lk_c")):
        _dev_f32(t, name)
    if w1.dim() != 2 or w1.shape[1] != C:
        raise ValueError(f"w1 must be [Ch, C] with C = {C}; got {tuple(w1.shape)}")
    Ch = int(w1.shape[0])
    if tuple(k_dw.shape) != (Ch, 3, 3) or tuple(w2.shape) != (C, Ch):
        raise ValueError("k_dw must be [Ch, 3, 3] and w2 [C, Ch]")
    if (b1 is not None and b1.numel() != Ch) or (b_dw is not None and b_dw.numel() != Ch) or \
            (b2 is not None and b2.numel() != C):
        raise ValueError("b1 and b_dw must hold Ch values, b2 C values")
    Ks, stride = _lk_checked(lk, int(Ca), None, None)
    if gen is not None:
        gen.check(int(Ca))
    if w_fuse.numel() != C * C or (b_fuse is not None and b_fuse.numel() != C):
        raise ValueError("w_fuse must be [C, C] and b_fuse [C]")
    if lk_c is not None and lk_c.numel() != Ca * Ca:
        raise ValueError("lk_c must be [Ca, Ca]")
    if out is None:
        out = torch.empty_like(f_in)
    if out.dtype != f_in.dtype or out.shape != f_in.shape or not out.is_contiguous():
        raise TypeError("out must match f_in in dtype and shape and be contiguous")
    _check(load_library().esc_residual_step_forward(
        _ptr(f_in), dt, N, C, H, W, Ch, _ptr(w1), _ptr(b1), _ptr(k_dw), _ptr(b_dw), _ptr(w2), _ptr(b2), int(Ca),
        _ptr(lk_c), _ptr(lk), Ks, stride, ctypes.byref(gen.c) if gen is not None else None, _ptr(w_fuse), _ptr(b_fuse),
        _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def new_dense_workspace(N: int, Ca: int, H: int, W: int, Ks: int, device="cuda", stream=None) -> torch.Tensor:
    """Allocate (with torch) and prepare a workspace for esc_convattn_dense_forward."""
    nbytes = int(load_library().esc_dense_workspace_bytes(N, Ca, H, W, Ks))
    if nbytes == 0:
        raise ValueError("bad shape for a workspace")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def convattn_dense_forward(x: torch.Tensor, Ca: int, lk_dense: torch.Tensor, workspace: torch.Tensor,
                           gen: Optional[GenParams] = None, dk_in: Optional[torch.Tensor] = None,
                           out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """esc_convattn_dense_forward.  lk_dense is [Ca, Ca, Ks, Ks], output channel first."""
    dt, (N, C, H, W) = _x_checked(x)
    _dev_f32(lk_dense, "lk_dense")
    if lk_dense.dim() != 4 or lk_dense.shape[0] != Ca or lk_dense.shape[1] != Ca or lk_dense.shape[2] != lk_dense.shape[3]:
        raise ValueError(f"lk_dense must be [Ca, Ca, Ks, Ks] with Ca = {Ca}; got {tuple(lk_dense.shape)}")
    Ks = int(lk_dense.shape[2])
    if gen is not None:
        gen.check(int(Ca))
    _dev_f32(dk_in, "dk_in")
    if dk_in is not None and dk_in.numel() != N * Ca * 9:
        raise ValueError("dk_in must hold [N, Ca, 3, 3] values")
    if out is None:
        out = torch.empty_like(x)
    if out.dtype != x.dtype or out.shape != x.shape or not out.is_contiguous():
        raise TypeError("out must match x in dtype and shape and be contiguous")
    _check(load_library().esc_convattn_dense_forward(
        _ptr(x), dt, N, C, H, W, int(Ca), _ptr(lk_dense), Ks, ctypes.byref(gen.c) if gen is not None else None,
        _ptr(dk_in), _ptr(out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
    return out


def new_backward_workspace(N: int, Ca: int, H: int, W: int, Ks: int, hidden: int, device="cuda", stream=None) -> torch.Tensor:
    """Allocate (with torch) and prepare a workspace for esc_convattn_backward."""
    nbytes = int(load_library().esc_backward_workspace_bytes(N, Ca, H, W, Ks, hidden))
    if nbytes == 0:
        raise ValueError("bad shape for a workspace")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    workspace_init(ws, stream)
    return ws


def convattn_backward(x: torch.Tensor, grad_out: torch.Tensor, Ca: int, lk: torch.Tensor, workspace: torch.Tensor,
                      gen: Optional[GenParams] = None, dk_in: Optional[torch.Tensor] = None, accumulate: bool = False,
                      grads: Optional[dict] = None, stream=None) -> dict:
    """esc_convattn_backward.  Returns a dict of device tensors: grad_x, grad_lk, grad_dk and, with an
    estimator, grad_w_up, grad_b_up (and grad_w_down, grad_b_down when hidden > 0).  `grads` may carry
    buffers to write into (required to make sense of accumulate=True)."""
    dt, (N, C, H, W) = _x_checked(x)
    if grad_out.dtype != x.dtype or grad_out.shape != x.shape or not grad_out.is_contiguous() or not grad_out.is_cuda:
        raise TypeError("grad_out must match x in dtype and shape and be a contiguous device tensor")
    Ks, stride = _lk_checked(lk, int(Ca), None, None)
    if gen is not None:
        gen.check(int(Ca))
    _dev_f32(dk_in, "dk_in")
    if dk_in is not None and dk_in.numel() != N * Ca * 9:
        raise ValueError("dk_in must hold [N, Ca, 3, 3] values")
    g = dict(grads or {})

    def need(name, make):  # (allocate only what the caller did not bring)
        if g.get(name) is None:
            g[name] = make()

    need("grad_x", lambda: torch.empty_like(x))
    need("grad_lk", lambda: torch.zeros_like(lk))
    need("grad_dk", lambda: torch.empty((N, Ca, 3, 3), dtype=torch.float32, device=x.device))
    gg = None
    if gen is not None:
        w_down, b_down, w_up, b_up = gen.tensors
        need("grad_w_up", lambda: torch.zeros_like(w_up))
        if b_up is not None:
            need("grad_b_up", lambda: torch.zeros_like(b_up))
        if gen.hidden > 0:
            need("grad_w_down", lambda: torch.zeros_like(w_down))
            if b_down is not None:
                need("grad_b_down", lambda: torch.zeros_like(b_down))
        gg = _GenGrads(_ptr(g.get("grad_w_down")), _ptr(g.get("grad_b_down")), _ptr(g.get("grad_w_up")),
                       _ptr(g.get("grad_b_up")))
    for k, v in g.items():
        if k != "grad_x":
            _dev_f32(v, k)
    _check(load_library().esc_convattn_backward(
        _ptr(x), _ptr(grad_out), dt, N, C, H, W, int(Ca), _ptr(lk), Ks, stride,
        ctypes.byref(gen.c) if gen is not None else None, _ptr(dk_in), _ptr(g["grad_x"]), _ptr(g["grad_lk"]),
        ctypes.byref(gg) if gg is not None else None, _ptr(g["grad_dk"]), int(bool(accumulate)),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))
    return g
