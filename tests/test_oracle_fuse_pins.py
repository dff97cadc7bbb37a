"""Pins of the oracle's point-wise steps (oracle/esc_oracle_fuse.c): Conv_fuse 1x1
(Eq. 4 line 4), the point-wise large-kernel factor LK^c (Eq. 5) and the residual of
Eq. 3 line 3, against things other than the oracle itself: identities and permutations
whose results are known exactly, a hand example, library 1x1 and grouped convolutions in
float64, the merged-kernel form of Eq. 5 through an FFT, and planted-mistake checks that
show a plausible slip (transposed weights, point-wise after instead of before, DK applied
to the unfiltered slice, GAP of the filtered slice) would be caught."""
import numpy as np
import pytest
import torch

from paper_2503_06671_amd import workloads as wk


def small(seed=0, N=2, C=7, H=9, W=11, Ca=3, Ks=5, dtype=wk.F32, **kw):
    return wk.make_random(seed, N, C, H, W, Ca, Ks, dtype=dtype, x_mean=0.3, **kw)


def rand_pointwise(seed, C, Ca):
    rng = np.random.default_rng(seed)
    w_fuse = (rng.standard_normal((C, C)) / np.sqrt(C)).astype(np.float32)
    b_fuse = (rng.standard_normal(C) * 0.1).astype(np.float32)
    lkc = (rng.standard_normal((Ca, Ca)) / np.sqrt(max(Ca, 1))).astype(np.float32)
    return w_fuse, b_fuse, lkc


def plain(oracle, wl, **kw):
    """The module without its point-wise steps (the part pinned elsewhere)."""
    return oracle.convattn_forward(wl.x, wl.Ca, wl.lk, wl.dtype, hidden=wl.hidden, w_up=wl.w_up, b_up=wl.b_up,
                                   w_down=wl.w_down, b_down=wl.b_down, want_out=False, **kw)


def fused(oracle, wl, w_fuse, **kw):
    return oracle.convattn_fused_forward(wl.x, wl.Ca, wl.lk, w_fuse, wl.dtype, hidden=wl.hidden, w_up=wl.w_up,
                                         b_up=wl.b_up, w_down=wl.w_down, b_down=wl.b_down, **kw)


# ------------------------------------------------------------------ Conv_fuse 1x1

def test_fuse_hand_example(oracle):
    # two channels, two pixels: out[co] = b[co] + w[co,0]*in[0] + w[co,1]*in[1] per pixel
    cat = np.array([[[[1.0, 2.0]], [[10.0, 20.0]]]])            # [1,2,1,2]
    w = np.array([[2.0, 0.5], [-1.0, 3.0]], np.float32)
    b = np.array([0.25, -4.0], np.float32)
    out = oracle.fuse_1x1(cat, w, b)
    assert out.tolist() == [[[[2 + 5 + 0.25, 4 + 10 + 0.25]], [[-1 + 30 - 4, -2 + 60 - 4]]]]
    assert oracle.fuse_1x1(cat, w).tolist() == [[[[7.0, 14.0]], [[29.0, 58.0]]]]


def test_fuse_matches_library_conv2d_float64(oracle):
    rng = np.random.default_rng(1)
    cat = rng.standard_normal((2, 6, 5, 7))
    w = rng.standard_normal((6, 6)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    want = torch.nn.functional.conv2d(torch.from_numpy(cat), torch.from_numpy(w).double()[:, :, None, None],
                                      torch.from_numpy(b).double()).numpy()
    np.testing.assert_allclose(oracle.fuse_1x1(cat, w, b), want, rtol=1e-13, atol=1e-13)


def test_identity_fuse_reproduces_the_module_without_it(oracle):
    # W_fuse = I, no bias, no LK^c: attention channels = F_res, identity channels = x, exactly
    wl = small(2)
    res_plain, dk_plain, _ = plain(oracle, wl)
    out, res, dk = fused(oracle, wl, np.eye(wl.C, dtype=np.float32))
    assert np.array_equal(res, res_plain) and np.array_equal(dk, dk_plain)
    assert np.array_equal(out[:, :wl.Ca], res_plain)
    assert np.array_equal(out[:, wl.Ca:], wl.x[:, wl.Ca:].astype(np.float64))


def test_permutation_fuse_permutes_channels_and_bias_adds(oracle):
    wl = small(3)
    perm = np.random.default_rng(4).permutation(wl.C)
    w = np.zeros((wl.C, wl.C), np.float32)
    w[np.arange(wl.C), perm] = 1.0                                  # out[co] = cat[perm[co]]
    b = np.arange(wl.C, dtype=np.float32) - 2.0
    base, _, _ = fused(oracle, wl, np.eye(wl.C, dtype=np.float32))
    out, _, _ = fused(oracle, wl, w, b_fuse=b)
    assert np.array_equal(out, base[:, perm] + b[None, :, None, None].astype(np.float64))


def test_transposed_fuse_weights_would_be_caught(oracle):
    # planted mistake: w[ci, co] instead of w[co, ci]
    wl = small(5)
    w, b, _ = rand_pointwise(6, wl.C, wl.Ca)
    out, _, _ = fused(oracle, wl, w, b_fuse=b)
    wrong, _, _ = fused(oracle, wl, np.ascontiguousarray(w.T), b_fuse=b)
    assert np.abs(out - wrong).max() > 1e-2 * np.abs(out).max()


def test_fused_forward_is_fuse_of_concat(oracle):
    # the whole call against its parts composed here: F_res from the plain module, the concat
    # written out, a float64 matrix product per pixel
    for dtype in (wk.F32, wk.BF16):
        wl = small(7, dtype=dtype)
        w, b, _ = rand_pointwise(8, wl.C, wl.Ca)
        res_plain, _, _ = plain(oracle, wl)
        cat = np.concatenate([res_plain, wl.x_as_f32()[:, wl.Ca:].astype(np.float64)], axis=1)
        want = np.einsum("oc,nchw->nohw", w.astype(np.float64), cat) + b.astype(np.float64)[None, :, None, None]
        out, _, _ = fused(oracle, wl, w, b_fuse=b)
        np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-12)


def test_residual_of_eq3_is_added_as_a_separate_tensor(oracle):
    for dtype in (wk.F32, wk.BF16):
        wl = small(9, dtype=dtype)
        w, b, _ = rand_pointwise(10, wl.C, wl.Ca)
        r = np.random.default_rng(11).standard_normal(wl.x.shape).astype(np.float32)
        r_st = wk.f32_to_bf16_bits(r) if dtype == wk.BF16 else r
        r_val = wk.bf16_bits_to_f32(r_st) if dtype == wk.BF16 else r
        out0, _, _ = fused(oracle, wl, w, b_fuse=b)
        out1, _, _ = fused(oracle, wl, w, b_fuse=b, residual=r_st)
        assert np.array_equal(out1, out0 + r_val.astype(np.float64))


# ------------------------------------------------------------------ LK^c (Eq. 5)

def test_pointwise_lkc_hand_example_and_library(oracle):
    x = np.zeros((1, 3, 1, 2), np.float32)
    x[0, 0, 0], x[0, 1, 0], x[0, 2, 0] = [1, 2], [10, 20], [100, 200]    # channel 2 is not in the slice
    lkc = np.array([[1.0, 1.0], [0.5, -1.0]], np.float32)
    pw = oracle.pointwise_lkc(x, 2, lkc)
    assert pw.tolist() == [[[[11.0, 22.0]], [[-9.5, -19.0]]]]
    rng = np.random.default_rng(12)
    x = rng.standard_normal((2, 6, 4, 5)).astype(np.float32)
    lkc = rng.standard_normal((4, 4)).astype(np.float32)
    want = torch.nn.functional.conv2d(torch.from_numpy(x[:, :4]).double(),
                                      torch.from_numpy(lkc).double()[:, :, None, None]).numpy()
    np.testing.assert_allclose(oracle.pointwise_lkc(x, 4, lkc), want, rtol=1e-13, atol=1e-13)
    xb = wk.f32_to_bf16_bits(x)
    want_b = np.einsum("oc,nchw->nohw", lkc.astype(np.float64), wk.bf16_bits_to_f32(xb)[:, :4].astype(np.float64))
    np.testing.assert_allclose(oracle.pointwise_lkc(xb, 4, lkc, wk.BF16), want_b, rtol=1e-13, atol=1e-13)


def test_identity_lkc_reproduces_the_depthwise_module(oracle):
    wl = small(13)
    res_plain, dk_plain, _ = plain(oracle, wl)
    _, res, dk = fused(oracle, wl, np.eye(wl.C, dtype=np.float32), lkc=np.eye(wl.Ca, dtype=np.float32))
    assert np.array_equal(res, res_plain) and np.array_equal(dk, dk_plain)


def fft_depthwise(img, ker):
    """Zero-padded 'same' cross-correlation of one plane with one odd kernel, through an FFT
    of the flipped kernel (library routine, shares nothing with the loops)."""
    H, W = img.shape
    K = ker.shape[0]
    p = (K - 1) // 2
    s = (H + K - 1, W + K - 1)
    full = np.fft.irfft2(np.fft.rfft2(img, s) * np.fft.rfft2(ker[::-1, ::-1], s), s)
    return full[p:p + H, p:p + W]


def test_eq5_merged_kernel_form_through_fft(oracle):
    # (F_att (*) LK^c) (*) (ZP(DK) + LK^s): point-wise product by a library einsum, then ONE
    # depth-wise convolution with the zero-padded DK added into LK^s, by FFT
    for Ks in (3, 7, 13):
        wl = small(14 + Ks, N=2, C=6, H=12, W=10, Ca=4, Ks=Ks)
        _, _, lkc = rand_pointwise(15, wl.C, wl.Ca)
        _, res, dk = fused(oracle, wl, np.eye(wl.C, dtype=np.float32), lkc=lkc)
        g = wl.x[:, :wl.Ca].astype(np.float64).mean(axis=(2, 3))
        dk_lib = (wl.w_up.astype(np.float64) @ g.T).T.reshape(wl.N, wl.Ca, 3, 3)   # GAP of the UNFILTERED slice
        np.testing.assert_allclose(dk, dk_lib, rtol=1e-12, atol=1e-14)
        pw = np.einsum("oc,nchw->nohw", lkc.astype(np.float64), wl.x[:, :wl.Ca].astype(np.float64))
        p = (Ks - 1) // 2
        for n in range(wl.N):
            for c in range(wl.Ca):
                merged = wl.lk[c].astype(np.float64).copy()
                merged[p - 1:p + 2, p - 1:p + 2] += dk_lib[n, c]
                np.testing.assert_allclose(res[n, c], fft_depthwise(pw[n, c], merged), rtol=1e-10, atol=1e-10)


def test_lkc_against_library_grouped_convolution(oracle):
    # F_pw by a library 1x1 conv2d, then library grouped convolutions for LK^s and DK
    wl = small(30, N=2, C=5, H=8, W=9, Ca=3, Ks=5)
    _, _, lkc = rand_pointwise(31, wl.C, wl.Ca)
    dk = np.random.default_rng(32).standard_normal((wl.N, wl.Ca, 3, 3))
    _, res, _ = oracle.convattn_fused_forward(wl.x, wl.Ca, wl.lk, np.eye(wl.C, dtype=np.float32), lkc=lkc, dk_in=dk)
    conv = torch.nn.functional.conv2d
    pw = conv(torch.from_numpy(wl.x[:, :wl.Ca]).double(), torch.from_numpy(lkc).double()[:, :, None, None])
    a = conv(pw, torch.from_numpy(wl.lk).double()[:, None], padding=2, groups=wl.Ca)
    for n in range(wl.N):
        b = conv(pw[n:n + 1], torch.from_numpy(dk[n])[:, None], padding=1, groups=wl.Ca)
        np.testing.assert_allclose(res[n], (a[n] + b[0]).numpy(), rtol=1e-12, atol=1e-12)


def test_order_of_pointwise_and_depthwise_is_pinned(oracle):
    # With ONE filter shared by all channels and DK = 0 a channel mix commutes with the
    # depth-wise convolution; with a filter per channel it does not.  So the oracle's order
    # (point-wise first, Eq. 5) is visible: it equals "mix afterwards" only in the shared case.
    wl = small(33, N=1, C=4, H=10, W=9, Ca=3, Ks=5)
    _, _, lkc = rand_pointwise(34, wl.C, wl.Ca)
    eye = np.eye(wl.C, dtype=np.float32)
    mix = lambda t: np.einsum("oc,nchw->nohw", lkc.astype(np.float64), t)
    shared = wl.lk[1]
    _, res_first, _ = oracle.convattn_fused_forward(wl.x, wl.Ca, shared, eye, lkc=lkc)
    res_plain, _, _ = oracle.convattn_forward(wl.x, wl.Ca, shared, want_out=False)
    np.testing.assert_allclose(res_first, mix(res_plain), rtol=1e-12, atol=1e-12)
    _, res_first, _ = oracle.convattn_fused_forward(wl.x, wl.Ca, wl.lk, eye, lkc=lkc)
    res_plain, _, _ = oracle.convattn_forward(wl.x, wl.Ca, wl.lk, want_out=False)
    assert np.abs(res_first - mix(res_plain)).max() > 1e-2 * np.abs(res_first).max()


def test_dk_acts_on_the_filtered_slice_but_comes_from_the_unfiltered_one(oracle):
    # Eq. 5 applies ZP(DK) + LK^s to F_att (*) LK^c; Eq. 4 line 2 estimates DK from GAP(F_att).
    # LK = 0 isolates the DK term.  Planted alternatives (DK on the unfiltered slice; GAP of the
    # filtered slice) must differ from the oracle.
    wl = small(35, N=2, C=5, H=8, W=9, Ca=3, Ks=3)
    _, _, lkc = rand_pointwise(36, wl.C, wl.Ca)
    zero_lk = np.zeros_like(wl.lk)
    eye = np.eye(wl.C, dtype=np.float32)
    _, res, dk = oracle.convattn_fused_forward(wl.x, wl.Ca, zero_lk, eye, lkc=lkc, w_up=wl.w_up)
    x64 = wl.x[:, :wl.Ca].astype(np.float64)
    pw = np.einsum("oc,nchw->nohw", lkc.astype(np.float64), x64)
    dk_unfiltered = (wl.w_up.astype(np.float64) @ x64.mean(axis=(2, 3)).T).T.reshape(2, 3, 3, 3)
    dk_filtered = (wl.w_up.astype(np.float64) @ pw.mean(axis=(2, 3)).T).T.reshape(2, 3, 3, 3)
    np.testing.assert_allclose(dk, dk_unfiltered, rtol=1e-12, atol=1e-14)
    assert np.abs(dk - dk_filtered).max() > 1e-2 * np.abs(dk).max()
    conv = lambda src, k: np.stack([[fft_depthwise(src[n, c], np.pad(k[n, c], 0)) for c in range(3)] for n in range(2)])
    np.testing.assert_allclose(res, conv(pw, dk_unfiltered), rtol=1e-10, atol=1e-10)
    assert np.abs(res - conv(x64, dk_unfiltered)).max() > 1e-2 * np.abs(res).max()


def test_fused_forward_scaling_law(oracle):
    # bias-free single-layer estimator and bias-free fuse: f(a x) = a L(x) + a^2 Q(x), with
    # L the LK part and Q the DK part, through LK^c and Conv_fuse alike (both linear)
    wl = small(37, N=1, C=5, H=8, W=9, Ca=3, Ks=5)
    w, _, lkc = rand_pointwise(38, wl.C, wl.Ca)
    f = lambda x, lk: oracle.convattn_fused_forward(x, wl.Ca, lk, w, lkc=lkc, w_up=wl.w_up)[0]
    a = np.float32(2.0)
    L = oracle.convattn_fused_forward(wl.x, wl.Ca, wl.lk, w, lkc=lkc)[0]          # DK = 0: linear part (incl. identity channels)
    Q = f(wl.x, wl.lk) - L
    np.testing.assert_allclose(f(a * wl.x, wl.lk), 2.0 * L + 4.0 * Q, rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("Ca", [0, 4])
def test_fused_forward_degenerate_slices(oracle, Ca):
    # C_a = 0: a plain 1x1 convolution of x; C_a = C: no identity channels
    wl = wk.make_random(39, 2, 4, 6, 7, Ca, 3, x_mean=0.2)
    w, b, lkc = rand_pointwise(40, 4, Ca)
    out, _, _ = oracle.convattn_fused_forward(wl.x, Ca, wl.lk, w, b_fuse=b, lkc=lkc if Ca else None,
                                              w_up=wl.w_up if Ca else None)
    if Ca == 0:
        want = np.einsum("oc,nchw->nohw", w.astype(np.float64), wl.x.astype(np.float64)) + b.astype(np.float64)[None, :, None, None]
        np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-12)
    else:
        res = oracle.convattn_fused_forward(wl.x, Ca, wl.lk, np.eye(4, dtype=np.float32), lkc=lkc, w_up=wl.w_up)[1]
        want = np.einsum("oc,nchw->nohw", w.astype(np.float64), res) + b.astype(np.float64)[None, :, None, None]
        np.testing.assert_allclose(out, want, rtol=1e-12, atol=1e-12)
