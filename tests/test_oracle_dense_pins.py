"""Pins of the oracle's dense large-kernel convolution (oracle/esc_oracle_dense.c; the LK
of the paper's main variants, Sec. 3, Eq. 4 line 3) against things other than itself: a
diagonal kernel reduces to the depth-wise oracle, single-entry kernels shift one input
channel into one output channel, a library dense convolution in float64, an FFT per
channel pair, the 1x1 case is a matrix product, and a planted mistake (input and output
channel swapped) is shown to differ."""
import numpy as np
import pytest
import torch

from paper_2503_06671_amd import workloads as wk


def rand_case(seed, N=2, C=6, H=9, W=11, Ca=4, Ks=5, dtype=wk.F32):
    wl = wk.make_random(seed, N, C, H, W, Ca, Ks, dtype=dtype, x_mean=0.3)
    rng = np.random.default_rng(seed + 1000)
    lk = (rng.standard_normal((Ca, Ca, Ks, Ks)) / (Ks * np.sqrt(max(Ca, 1)))).astype(np.float32)
    return wl, lk


def test_diagonal_dense_kernel_is_the_depthwise_one(oracle):
    wl, lk = rand_case(1)
    diag = np.zeros_like(lk)
    for c in range(wl.Ca):
        diag[c, c] = wl.lk[c]
    want = oracle.lk_conv(wl.x, wl.Ca, wl.lk)
    assert np.array_equal(oracle.dense_lk_conv(wl.x, wl.Ca, diag), want)


def test_single_entry_kernel_shifts_one_channel_into_another(oracle):
    # lk[co=2, ci=1, i0=1, j0=3] = 1 with Ks = 5 (p = 2): out[2][y,x] = x[1][y-1, x+1], zero elsewhere
    wl, lk = rand_case(2, N=1, H=8, W=9)
    one = np.zeros_like(lk)
    one[2, 1, 1, 3] = 1.0
    res = oracle.dense_lk_conv(wl.x, wl.Ca, one)
    want = np.zeros((8, 9))
    want[1:, :-1] = wl.x[0, 1, :-1, 1:]
    assert np.array_equal(res[0, 2], want)
    assert not res[0, [0, 1, 3]].any()


@pytest.mark.parametrize("dtype", [wk.F32, wk.BF16])
@pytest.mark.parametrize("Ks", [1, 3, 13])
def test_dense_conv_matches_library_conv2d_float64(oracle, dtype, Ks):
    wl, lk = rand_case(3 + Ks, H=15 if Ks == 13 else 7, W=10, Ks=Ks, dtype=dtype)
    xa = torch.from_numpy(wl.x_as_f32()[:, :wl.Ca]).double()
    want = torch.nn.functional.conv2d(xa, torch.from_numpy(lk).double(), padding=(Ks - 1) // 2).numpy()
    np.testing.assert_allclose(oracle.dense_lk_conv(wl.x, wl.Ca, lk, dtype), want, rtol=1e-12, atol=1e-13)


def test_dense_conv_through_fft_per_channel_pair(oracle):
    wl, lk = rand_case(20, N=1, C=3, H=12, W=10, Ca=3, Ks=7)
    p = 3
    s = (12 + 6, 10 + 6)
    want = np.zeros((3, 12, 10))
    for co in range(3):
        for ci in range(3):
            full = np.fft.irfft2(np.fft.rfft2(wl.x[0, ci].astype(np.float64), s) *
                                 np.fft.rfft2(lk[co, ci, ::-1, ::-1].astype(np.float64), s), s)
            want[co] += full[p:p + 12, p:p + 10]
    np.testing.assert_allclose(oracle.dense_lk_conv(wl.x, 3, lk)[0], want, rtol=1e-10, atol=1e-11)


def test_one_by_one_dense_kernel_is_a_matrix_product(oracle):
    wl, lk = rand_case(21, Ks=1)
    want = np.einsum("oc,nchw->nohw", lk[:, :, 0, 0].astype(np.float64), wl.x[:, :wl.Ca].astype(np.float64))
    np.testing.assert_allclose(oracle.dense_lk_conv(wl.x, wl.Ca, lk), want, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(oracle.dense_lk_conv(wl.x, wl.Ca, lk), oracle.pointwise_lkc(wl.x, wl.Ca, lk[:, :, 0, 0]),
                               rtol=1e-13, atol=1e-14)


def test_swapped_channel_roles_would_be_caught(oracle):
    wl, lk = rand_case(22)
    res = oracle.dense_lk_conv(wl.x, wl.Ca, lk)
    wrong = oracle.dense_lk_conv(wl.x, wl.Ca, np.ascontiguousarray(lk.transpose(1, 0, 2, 3)))
    assert np.abs(res - wrong).max() > 1e-2 * np.abs(res).max()


@pytest.mark.parametrize("dtype", [wk.F32, wk.BF16])
def test_dense_forward_is_the_sum_of_its_parts(oracle, dtype):
    # F_res = dense LK term + depth-wise DK term (DK from the estimator on GAP(F_att)); identity
    # channels are bit copies; the estimator's DK equals the depth-wise module's
    wl, lk = rand_case(23, dtype=dtype)
    res, dk, out = oracle.convattn_dense_forward(wl.x, wl.Ca, lk, dtype, w_up=wl.w_up)
    _, dk_plain, out_plain = oracle.forward_workload(wl)
    assert np.array_equal(dk, dk_plain)
    want = oracle.dense_lk_conv(wl.x, wl.Ca, lk, dtype) + oracle.dk_conv(wl.x, wl.Ca, dk, dtype)
    assert np.array_equal(res, want)
    assert np.array_equal(out[:, wl.Ca:], wl.x[:, wl.Ca:]) and np.array_equal(out[:, wl.Ca:], out_plain[:, wl.Ca:])
    stored = wk.bf16_bits_to_f32(out[:, :wl.Ca]) if dtype == wk.BF16 else out[:, :wl.Ca]
    np.testing.assert_allclose(stored, res, rtol=2 ** -8 if dtype == wk.BF16 else 2 ** -23, atol=1e-30)
    # DK given, and no DK
    dk_in = np.random.default_rng(24).standard_normal((wl.N, wl.Ca, 3, 3))
    res2, _, _ = oracle.convattn_dense_forward(wl.x, wl.Ca, lk, dtype, dk_in=dk_in, want_out=False)
    assert np.array_equal(res2, oracle.dense_lk_conv(wl.x, wl.Ca, lk, dtype) + oracle.dk_conv(wl.x, wl.Ca, dk_in, dtype))
    res3, _, _ = oracle.convattn_dense_forward(wl.x, wl.Ca, lk, dtype, want_out=False)
    assert np.array_equal(res3, oracle.dense_lk_conv(wl.x, wl.Ca, lk, dtype))


def test_dense_forward_with_diagonal_kernel_equals_the_depthwise_forward(oracle):
    wl, lk = rand_case(25)
    diag = np.zeros_like(lk)
    for c in range(wl.Ca):
        diag[c, c] = wl.lk[c]
    res, dk, out = oracle.convattn_dense_forward(wl.x, wl.Ca, diag, w_up=wl.w_up)
    res_p, dk_p, out_p = oracle.forward_workload(wl)
    assert np.array_equal(res, res_p) and np.array_equal(dk, dk_p) and np.array_equal(out, out_p)
