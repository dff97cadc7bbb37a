"""Pins of the backward oracle (oracle/esc_oracle_backward.c: gradients of the depth-wise
ConvAttn forward, Eq. 4 lines 1-4 without Conv_fuse) against things other than itself:
library automatic differentiation in float64 of the forward composed from library
operators, exact central differences of the FORWARD oracle (the module is a quadratic
polynomial in x and linear in LK when the estimator is the bias-free linear layer, so
central differences are exact on inputs chosen to be exactly representable), closed
forms for delta kernels, and the shared-filter case."""
import numpy as np
import pytest
import torch

from paper_2503_06671_amd import workloads as wk


def case(seed, N=2, C=5, H=7, W=9, Ca=3, Ks=5, hidden=0, bias=False, dtype=wk.F32):
    wl = wk.make_random(seed, N, C, H, W, Ca, Ks, dtype=dtype, hidden=hidden, bias=bias, x_mean=0.3)
    go = np.random.default_rng(seed + 5000).standard_normal((N, C, H, W)).astype(np.float32)
    if dtype == wk.BF16:
        go = wk.f32_to_bf16_bits(go)
    return wl, go


def backward(oracle, wl, go, **kw):
    return oracle.convattn_backward(wl.x, go, wl.Ca, wl.lk, wl.dtype, hidden=wl.hidden, w_up=wl.w_up, b_up=wl.b_up,
                                    w_down=wl.w_down, b_down=wl.b_down, **kw)


def torch_grads(wl, go):
    """The forward composed from library operators in float64, differentiated by the library."""
    f64 = lambda a: None if a is None else torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True)
    x = f64(wl.x_as_f32())
    lk, w_up, b_up, w_down, b_down = f64(wl.lk), f64(wl.w_up), f64(wl.b_up), f64(wl.w_down), f64(wl.b_down)
    N, C, H, W = x.shape
    Ca, Ks = wl.Ca, wl.Ks
    xa = x[:, :Ca]
    g = xa.mean(dim=(2, 3))
    t = g
    if wl.hidden > 0:
        t = torch.nn.functional.gelu(torch.nn.functional.linear(g, w_down, b_down))
    d = torch.nn.functional.linear(t, w_up, b_up)
    dk = d.reshape(N, Ca, 3, 3)
    a = torch.nn.functional.conv2d(xa, lk[:, None], padding=(Ks - 1) // 2, groups=Ca)
    b = torch.nn.functional.conv2d(xa.reshape(1, N * Ca, H, W), dk.reshape(N * Ca, 1, 3, 3), padding=1,
                                   groups=N * Ca).reshape(N, Ca, H, W)
    out = torch.cat([a + b, x[:, Ca:]], dim=1)
    gof = wk.bf16_bits_to_f32(go) if wl.dtype == wk.BF16 else go
    (out * torch.tensor(gof.astype(np.float64))).sum().backward()
    grads = {"dx": x.grad, "dlk": lk.grad, "dw_up": w_up.grad}
    if b_up is not None:
        grads["db_up"] = b_up.grad
    if wl.hidden > 0:
        grads["dw_down"] = w_down.grad
        if b_down is not None:
            grads["db_down"] = b_down.grad
    return {k: v.numpy() for k, v in grads.items()}


@pytest.mark.parametrize("hidden,bias,dtype,Ks", [(0, False, wk.F32, 5), (0, True, wk.F32, 1), (4, True, wk.F32, 7),
                                                  (8, False, wk.BF16, 3), (0, False, wk.BF16, 13)])
def test_backward_matches_library_autodiff(oracle, hidden, bias, dtype, Ks):
    wl, go = case(10 + hidden + Ks, H=9 if Ks < 13 else 15, Ks=Ks, hidden=hidden, bias=bias, dtype=dtype)
    got = backward(oracle, wl, go)
    want = torch_grads(wl, go)
    for k, v in want.items():
        np.testing.assert_allclose(got[k], v, rtol=1e-10, atol=1e-11, err_msg=k)
    if bias:
        assert "db_up" in want and (hidden == 0 or "db_down" in want)


def quantised(a, step=2.0 ** -6):
    return (np.round(a / step) * step).astype(np.float32)


def test_backward_against_exact_central_differences_of_the_forward_oracle(oracle):
    # bias-free single-layer estimator: out is a quadratic polynomial in x and linear in LK and in
    # W_up, so (f(v + h e) - f(v - h e)) / 2h is the exact directional derivative.  All values are
    # multiples of 2^-6 and h = 2^-3, so every perturbed input is exact in float32 and the forward
    # oracle (float64 inside) commits no rounding that matters.
    wl, go = case(30, N=2, C=4, H=6, W=7, Ca=2, Ks=3)
    wl.x, wl.lk, wl.w_up, go = quantised(wl.x), quantised(wl.lk), quantised(wl.w_up), quantised(go)
    got = backward(oracle, wl, go)
    h = np.float32(2.0 ** -3)
    rng = np.random.default_rng(31)

    def loss(x, lk, w_up):
        res, _, _ = oracle.convattn_forward(x, wl.Ca, lk, hidden=0, w_up=w_up, want_out=False)
        full = np.concatenate([res, x[:, wl.Ca:].astype(np.float64)], axis=1)
        return float((full * go.astype(np.float64)).sum())

    for name, base in (("dx", wl.x), ("dlk", wl.lk), ("dw_up", wl.w_up)):
        for _ in range(6):
            e = rng.integers(-1, 2, size=base.shape).astype(np.float32)
            args = {"dx": (wl.x, wl.lk, wl.w_up), "dlk": (wl.x, wl.lk, wl.w_up), "dw_up": (wl.x, wl.lk, wl.w_up)}[name]
            plus = [a.copy() for a in args]
            minus = [a.copy() for a in args]
            idx = {"dx": 0, "dlk": 1, "dw_up": 2}[name]
            plus[idx] = (base + h * e).astype(np.float32)
            minus[idx] = (base - h * e).astype(np.float32)
            fd = (loss(*plus) - loss(*minus)) / (2.0 * float(h))
            want = float((got[name] * e.astype(np.float64)).sum())
            assert abs(fd - want) <= 1e-9 * max(1.0, abs(want)), (name, fd, want)


def test_delta_kernel_closed_forms(oracle):
    # LK = centre delta, DK = 0: out_att = x_att, so dx_att = go_att exactly, dLK[c] is the
    # correlation of go with x, whose centre entry is sum(go * x) and whose (p, p+1) entry is
    # sum over y, x of go[y, x] * x[y, x + 1]
    wl, go = case(40, N=1, C=3, H=6, W=8, Ca=2, Ks=5)
    wl.lk[:] = 0
    wl.lk[:, 2, 2] = 1.0
    got = oracle.convattn_backward(wl.x, go, wl.Ca, wl.lk)
    assert np.array_equal(got["dx"], go.astype(np.float64))
    x64, g64 = wl.x.astype(np.float64), go.astype(np.float64)
    for c in range(2):
        np.testing.assert_allclose(got["dlk"][c, 2, 2], (g64[0, c] * x64[0, c]).sum(), rtol=1e-13)
        np.testing.assert_allclose(got["dlk"][c, 2, 3], (g64[0, c, :, :-1] * x64[0, c, :, 1:]).sum(), rtol=1e-13)
        np.testing.assert_allclose(got["dlk"][c, 0, 2], (g64[0, c, 2:, :] * x64[0, c, :-2, :]).sum(), rtol=1e-13)
        # dDK is the centre 3 x 3 of the same correlation
        np.testing.assert_allclose(got["ddk"][0, c], got["dlk"][c, 1:4, 1:4], rtol=1e-13)


def test_shared_filter_gradient_sums_over_channels(oracle):
    wl, go = case(41, Ca=3, Ks=5)
    shared = wl.lk[1].copy()
    per_channel = oracle.convattn_backward(wl.x, go, wl.Ca, np.stack([shared] * 3))
    one = oracle.convattn_backward(wl.x, go, wl.Ca, shared)
    assert one["dlk"].shape == (5, 5)
    np.testing.assert_allclose(one["dlk"], per_channel["dlk"].sum(axis=0), rtol=1e-13, atol=1e-13)
    assert np.array_equal(one["dx"], per_channel["dx"])


def test_given_dk_has_no_estimator_path(oracle):
    # DK given: no gradient flows through GAP, dx is the two transposed convolutions alone
    wl, go = case(42)
    dk = np.random.default_rng(43).standard_normal((wl.N, wl.Ca, 3, 3))
    got = oracle.convattn_backward(wl.x, go, wl.Ca, wl.lk, dk_in=dk)
    assert not got["dg"].any() and "dw_up" not in got
    xa = torch.tensor(wl.x[:, :wl.Ca].astype(np.float64), requires_grad=True)
    N, Ca, H, W = xa.shape
    a = torch.nn.functional.conv2d(xa, torch.tensor(wl.lk.astype(np.float64))[:, None], padding=2, groups=Ca)
    b = torch.nn.functional.conv2d(xa.reshape(1, N * Ca, H, W), torch.tensor(dk).reshape(N * Ca, 1, 3, 3), padding=1,
                                   groups=N * Ca).reshape(N, Ca, H, W)
    ((a + b) * torch.tensor(go[:, :Ca].astype(np.float64))).sum().backward()
    np.testing.assert_allclose(got["dx"][:, :Ca], xa.grad.numpy(), rtol=1e-11, atol=1e-12)
    assert np.array_equal(got["dx"][:, Ca:], go[:, Ca:].astype(np.float64))
