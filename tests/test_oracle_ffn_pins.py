"""Pins of the oracle's ConvFFN (oracle/esc_oracle_ffn.c; Eq. 3 of the ESC paper names the
network, Sec. 3 fixes its kernel size at three) against things other than the oracle
itself: a hand example, table values of the normal distribution for the GELU, shifted
deltas and tap counts with closed forms, library convolutions and GELU in float64, and
planted-mistake checks."""
import math

import numpy as np
import pytest
import torch

from paper_2503_06671_amd import workloads as wk

F = torch.nn.functional


def library_convffn(x, p):
    """float64 library ops: 1x1 conv, erf-GELU, grouped 3x3 conv with padding 1, 1x1 conv."""
    t = lambda a: None if a is None else torch.from_numpy(np.asarray(a)).double()
    Ch = p["w1"].shape[0]
    u = F.gelu(F.conv2d(t(x), t(p["w1"])[:, :, None, None], t(p["b1"])))
    v = u + F.gelu(F.conv2d(u, t(p["k"])[:, None], t(p["bk"]), padding=1, groups=Ch))
    return F.conv2d(v, t(p["w2"])[:, :, None, None], t(p["b2"])).numpy()


def test_hand_example(oracle):
    # one channel in, one hidden, one out, a 1 x 3 image
    x = np.array([[[[1.0, -2.0, 0.5]]]], np.float32)
    w1, b1 = np.array([[2.0]], np.float32), np.array([0.5], np.float32)
    k = np.zeros((1, 3, 3), np.float32)
    k[0, 1, 0], k[0, 1, 1], k[0, 1, 2] = 1.0, -1.0, 3.0      # left, centre, right of the middle row
    bk = np.array([0.25], np.float32)
    w2, b2 = np.array([[-1.5]], np.float32), np.array([4.0], np.float32)
    g = lambda v: 0.5 * v * (1.0 + math.erf(v / math.sqrt(2.0)))
    u = [g(2.0 * v + 0.5) for v in (1.0, -2.0, 0.5)]
    d = [0.25 - u[0] + 3 * u[1], 0.25 + u[0] - u[1] + 3 * u[2], 0.25 + u[1] - u[2]]
    want = [4.0 - 1.5 * (u[i] + g(d[i])) for i in range(3)]
    got = oracle.convffn_forward(x, w1, k, w2, b1=b1, bk=bk, b2=b2)
    np.testing.assert_allclose(got.ravel(), want, rtol=1e-14, atol=1e-14)


def test_gelu_is_the_erf_form(oracle):
    # gelu(v) = v * Phi(v); Phi from the printed table of the normal distribution
    table = {0.5: 0.6914624613, 1.0: 0.8413447461, 2.0: 0.9772498681, -1.0: 0.1586552539}
    for v, phi in table.items():
        x = np.full((1, 1, 1, 1), v, np.float32)
        u = oracle.ffn_expand(x, np.ones((1, 1), np.float32))
        assert abs(u.item() - v * phi) < 2e-10, (v, u.item())
    # the tanh approximation differs from it by 1.5e-4 at v = 1: must not be that
    tanh1 = 0.5 * (1 + math.tanh(math.sqrt(2 / math.pi) * (1 + 0.044715)))
    u1 = oracle.ffn_expand(np.ones((1, 1, 1, 1), np.float32), np.ones((1, 1), np.float32)).item()
    assert abs(u1 - tanh1) > 1e-4


@pytest.mark.parametrize("i0,j0", [(0, 0), (0, 2), (1, 0), (2, 1), (1, 1)])
def test_branch_with_a_shifted_delta(oracle, i0, j0):
    # k = delta at (i0, j0): v[y, x] = u[y, x] + gelu(u[y + i0 - 1, x + j0 - 1]), zero outside
    rng = np.random.default_rng(3)
    u = rng.standard_normal((2, 3, 5, 7))
    k = np.zeros((3, 3, 3), np.float32)
    k[:, i0, j0] = 1.0
    sh = np.zeros_like(u)
    H, W = u.shape[2:]
    for y in range(H):
        for x in range(W):
            yy, xx = y + i0 - 1, x + j0 - 1
            if 0 <= yy < H and 0 <= xx < W:
                sh[:, :, y, x] = u[:, :, yy, xx]
    want = u + F.gelu(torch.from_numpy(sh)).numpy()
    np.testing.assert_allclose(oracle.ffn_dwbranch(u, k), want, rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("H,W", [(1, 1), (1, 5), (2, 2), (4, 6)])
def test_branch_tap_counts_at_the_border(oracle, H, W):
    # u = 1, k = 1: the depth-wise sum is the number of taps inside the image
    u = np.ones((1, 2, H, W))
    cnt = lambda L, t: min(t, 1) + min(L - 1 - t, 1) + 1
    want = np.empty((H, W))
    for y in range(H):
        for x in range(W):
            s = float(cnt(H, y) * cnt(W, x))
            want[y, x] = 1.0 + 0.5 * s * (1.0 + math.erf(s / math.sqrt(2.0)))
    got = oracle.ffn_dwbranch(u, np.ones((2, 3, 3), np.float32))
    np.testing.assert_allclose(got[0, 0], want, rtol=1e-14)
    np.testing.assert_allclose(got[0, 1], want, rtol=1e-14)


def test_zero_branch_leaves_two_linear_layers(oracle):
    # k = 0, bk = 0: gelu(0) = 0, so Y = W2 gelu(W1 x + b1) + b2
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, 5, 4, 6)).astype(np.float32)
    p = wk.make_ffn_params(40, 5, 9)
    p["k"][:] = 0
    p["bk"] = None
    h = F.gelu(torch.einsum("mc,nchw->nmhw", torch.from_numpy(p["w1"]).double(), torch.from_numpy(x).double())
               + torch.from_numpy(p["b1"]).double()[None, :, None, None])
    want = (torch.einsum("cm,nmhw->nchw", torch.from_numpy(p["w2"]).double(), h)
            + torch.from_numpy(p["b2"]).double()[None, :, None, None]).numpy()
    got = oracle.convffn_forward(x, p["w1"], p["k"], p["w2"], b1=p["b1"], b2=p["b2"])
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("bias", [True, False])
@pytest.mark.parametrize("shape", [(1, 3, 1, 1, 4), (2, 6, 7, 9, 12), (1, 8, 12, 5, 8), (3, 4, 2, 13, 5)])
def test_whole_network_matches_library_ops_in_float64(oracle, shape, bias):
    N, C, H, W, Ch = shape
    rng = np.random.default_rng(N * 100 + C)
    x = (rng.standard_normal((N, C, H, W)) + 0.2).astype(np.float32)
    p = wk.make_ffn_params(7 + C, C, Ch, bias=bias)
    got = oracle.convffn_forward(x, p["w1"], p["k"], p["w2"], b1=p["b1"], bk=p["bk"], b2=p["b2"])
    np.testing.assert_allclose(got, library_convffn(x, p), rtol=1e-12, atol=1e-12)


def test_whole_is_its_three_steps(oracle):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 4, 6, 5)).astype(np.float32)
    p = wk.make_ffn_params(50, 4, 7)
    u = oracle.ffn_expand(x, p["w1"], p["b1"])
    v = oracle.ffn_dwbranch(u, p["k"], p["bk"])
    y = oracle.ffn_project(v, p["w2"], p["b2"])
    got = oracle.convffn_forward(x, p["w1"], p["k"], p["w2"], b1=p["b1"], bk=p["bk"], b2=p["b2"])
    assert np.array_equal(got, y)


def test_projection_with_a_permutation_permutes_channels(oracle):
    rng = np.random.default_rng(6)
    v = rng.standard_normal((1, 4, 3, 3))
    perm = [2, 0, 3, 1]
    w2 = np.zeros((4, 4), np.float32)
    for co, ci in enumerate(perm):
        w2[co, ci] = 1.0
    assert np.array_equal(oracle.ffn_project(v, w2), v[:, perm])


def test_bf16_storage_is_widened_exactly(oracle):
    rng = np.random.default_rng(8)
    xf = rng.standard_normal((1, 3, 4, 5)).astype(np.float32)
    bits = wk.f32_to_bf16_bits(xf)
    wide = (bits.astype(np.uint32) << 16).view(np.float32)
    p = wk.make_ffn_params(80, 3, 6)
    a = oracle.convffn_forward(bits, p["w1"], p["k"], p["w2"], wk.BF16, b1=p["b1"], bk=p["bk"], b2=p["b2"])
    b = oracle.convffn_forward(wide, p["w1"], p["k"], p["w2"], wk.F32, b1=p["b1"], bk=p["bk"], b2=p["b2"])
    assert np.array_equal(a, b)


def test_images_are_independent(oracle):
    rng = np.random.default_rng(9)
    x = rng.standard_normal((3, 4, 5, 6)).astype(np.float32)
    p = wk.make_ffn_params(90, 4, 8)
    whole = oracle.convffn_forward(x, p["w1"], p["k"], p["w2"], b1=p["b1"], bk=p["bk"], b2=p["b2"])
    for n in range(3):
        one = oracle.convffn_forward(x[n:n + 1], p["w1"], p["k"], p["w2"], b1=p["b1"], bk=p["bk"], b2=p["b2"])
        assert np.array_equal(whole[n:n + 1], one)


def test_planted_mistakes_would_be_caught(oracle):
    """What a plausible slip would give differs from the oracle far beyond rounding."""
    rng = np.random.default_rng(10)
    x = rng.standard_normal((1, 4, 6, 7)).astype(np.float32)
    p = wk.make_ffn_params(100, 4, 4)   # square, so that a transposed weight has the right shape
    ref = oracle.convffn_forward(x, p["w1"], p["k"], p["w2"], b1=p["b1"], bk=p["bk"], b2=p["b2"])
    scale = np.abs(ref).max()
    slips = {
        "w1 transposed": dict(p, w1=np.ascontiguousarray(p["w1"].T)),
        "w2 transposed": dict(p, w2=np.ascontiguousarray(p["w2"].T)),
        "kernel flipped (convolution instead of correlation)": dict(p, k=np.ascontiguousarray(p["k"][:, ::-1, ::-1])),
        "kernel transposed": dict(p, k=np.ascontiguousarray(p["k"].transpose(0, 2, 1))),
    }
    for name, q in slips.items():
        got = library_convffn(x, q)
        assert np.abs(got - ref).max() > 1e-3 * scale, name
    # no skip around the branch, no GELU on the branch, no GELU after the first layer
    t = lambda a: torch.from_numpy(np.asarray(a)).double()
    u = F.gelu(F.conv2d(t(x), t(p["w1"])[:, :, None, None], t(p["b1"])))
    d = F.conv2d(u, t(p["k"])[:, None], t(p["bk"]), padding=1, groups=4)
    proj = lambda v: F.conv2d(v, t(p["w2"])[:, :, None, None], t(p["b2"])).numpy()
    for name, v in {"no skip": F.gelu(d), "no GELU on the branch": u + d}.items():
        assert np.abs(proj(v) - ref).max() > 1e-3 * scale, name
