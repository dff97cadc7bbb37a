"""GPU parity of esc_convattn_fused_forward (the module with Conv_fuse, Eq. 4 line 4;
optionally LK^c in front of the depth-wise kernels, Eq. 5; optionally the residual of
Eq. 3 line 3) against the CPU oracle, through the C ABI.

Bars: every output element within 1e-5 (fp32 storage) / 2e-2 (bf16 storage) of the
oracle's unrounded float64 result, normwise and elementwise as for the attention slice
of the plain forward (gpu_util.assert_att_close)."""
import numpy as np
import pytest
import torch

from paper_2503_06671_amd import binding, workloads as wk
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

F32, BF16 = wk.F32, wk.BF16


def pointwise_weights(seed, C, Ca, bias=True):
    rng = np.random.default_rng(seed)
    w_fuse = (rng.standard_normal((C, C)) / np.sqrt(C)).astype(np.float32)
    b_fuse = (rng.standard_normal(C) * 0.1).astype(np.float32) if bias else None
    lkc = (rng.standard_normal((Ca, Ca)) / np.sqrt(max(Ca, 1))).astype(np.float32)
    return w_fuse, b_fuse, lkc


def residual_for(wl, seed):
    r = np.random.default_rng(seed).standard_normal(wl.x.shape).astype(np.float32)
    return wk.f32_to_bf16_bits(r) if wl.dtype == BF16 else r


def out_as_f64(out_np, wl):
    return (wk.bf16_bits_to_f32(out_np) if wl.dtype == BF16 else out_np).astype(np.float64)


def run_fused(wl, w_fuse, b_fuse=None, lkc=None, residual=None, use_gen=True, dk_in=None):
    x = gu.to_dev_x(wl.x, wl.dtype)
    ws = binding.new_fused_workspace(wl.N, wl.Ca, wl.H, wl.W, x.dtype, lkc is not None)
    out = torch.full_like(x, float("nan"))
    binding.convattn_fused_forward(
        x, wl.Ca, gu.dev(wl.lk), gu.dev(w_fuse), ws, b_fuse=gu.dev(b_fuse), lk_c=gu.dev(lkc),
        residual=None if residual is None else gu.to_dev_x(residual, wl.dtype),
        gen=gu.gen_params(wl) if use_gen and wl.Ca > 0 else None, dk_in=gu.dev(dk_in), out=out)
    assert binding.workspace_errors(ws) == 0
    torch.cuda.synchronize()
    return gu.out_to_np(out, wl.dtype)


def check_fused(wl, oracle, w_fuse, b_fuse=None, lkc=None, residual=None, what=None):
    what = what or wl.name
    print(f"[case] fused {what} lkc={lkc is not None} bias={b_fuse is not None} residual={residual is not None}", flush=True)
    ref, _, _ = oracle.convattn_fused_forward(
        wl.x, wl.Ca, wl.lk, w_fuse, wl.dtype, b_fuse=b_fuse, lkc=lkc, residual=residual, hidden=wl.hidden,
        w_up=wl.w_up if wl.Ca > 0 else None, b_up=wl.b_up, w_down=wl.w_down, b_down=wl.b_down)
    got = run_fused(wl, w_fuse, b_fuse, lkc, residual)
    return gu.assert_att_close(out_as_f64(got, wl), ref, wl.dtype, what)


# ------------------------------------------------------------------ small and ragged shapes

@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("with_lkc", [False, True])
@pytest.mark.parametrize("N,C,H,W,Ca,Ks", [
    (2, 7, 45, 70, 3, 13),     # odd channel count (a padded channel pair), ragged tiles
    (1, 6, 9, 11, 4, 5),       # odd plane size: element-wise accesses
    (3, 48, 40, 72, 16, 13),   # the FLOPs-lean variant's width
    (2, 70, 30, 50, 16, 7),    # more than 64 channels: two passes over the inputs
    (1, 5, 1, 1, 2, 3),        # a single pixel
    (40, 8, 20, 24, 4, 3),     # many images, even planes: two pixels per lane
])
def test_fused_small_shapes(oracle, dtype, with_lkc, N, C, H, W, Ca, Ks):
    wl = wk.make_random(700 + C + H, N, C, H, W, Ca, Ks, dtype=dtype, x_mean=0.3)
    w_fuse, b_fuse, lkc = pointwise_weights(701 + C, C, Ca)
    check_fused(wl, oracle, w_fuse, b_fuse, lkc if with_lkc else None, residual_for(wl, 702))


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_fused_without_optional_inputs(oracle, dtype):
    wl = wk.make_random(710, 2, 9, 33, 40, 4, 9, dtype=dtype, x_mean=0.3)
    w_fuse, _, _ = pointwise_weights(711, wl.C, wl.Ca)
    check_fused(wl, oracle, w_fuse)


@pytest.mark.parametrize("Ca", [0, 6])
def test_fused_degenerate_slices(oracle, Ca):
    # C_a = 0: a plain 1x1 convolution of x; C_a = C: no identity channels
    wl = wk.make_random(720 + Ca, 2, 6, 20, 26, Ca, 5, x_mean=0.3)
    w_fuse, b_fuse, lkc = pointwise_weights(721, 6, Ca)
    check_fused(wl, oracle, w_fuse, b_fuse, lkc if Ca else None, residual_for(wl, 722))


def test_fused_two_layer_estimator_and_given_dk(oracle):
    wl = wk.make_random(730, 2, 20, 40, 72, 16, 13, hidden=8, bias=True, x_mean=0.5)
    w_fuse, b_fuse, lkc = pointwise_weights(731, wl.C, wl.Ca)
    check_fused(wl, oracle, w_fuse, b_fuse, lkc)
    # DK given by the caller instead of the estimator
    dk = np.random.default_rng(732).standard_normal((2, 16, 3, 3)).astype(np.float32)
    ref, _, _ = oracle.convattn_fused_forward(wl.x, wl.Ca, wl.lk, w_fuse, b_fuse=b_fuse, lkc=lkc, dk_in=dk)
    got = run_fused(wl, w_fuse, b_fuse, lkc, use_gen=False, dk_in=dk)
    gu.assert_att_close(got.astype(np.float64), ref, F32, "given dk")


# ------------------------------------------------------------------ exact special cases

@pytest.mark.parametrize("dtype", [F32, BF16])
def test_identity_pointwise_weights_reproduce_the_plain_forward_bit_for_bit(dtype):
    # W_fuse = I and LK^c = I: products with 1 and sums with 0 are exact, so the fused call
    # must return the plain forward's output, bits and all
    wl = wk.make_random(740, 2, 6, 40, 72, 4, 13, dtype=dtype, x_mean=0.4)
    plain = gu.run_forward(wl)
    eye_c, eye_a = np.eye(wl.C, dtype=np.float32), np.eye(wl.Ca, dtype=np.float32)
    assert np.array_equal(run_fused(wl, eye_c).view(np.uint8), plain.view(np.uint8))
    assert np.array_equal(run_fused(wl, eye_c, lkc=eye_a).view(np.uint8), plain.view(np.uint8))


def test_permutation_fuse_permutes_the_plain_forward():
    wl = wk.make_random(741, 1, 70, 24, 40, 16, 5, x_mean=0.4)
    plain = gu.run_forward(wl)
    perm = np.random.default_rng(742).permutation(wl.C)
    w = np.zeros((wl.C, wl.C), np.float32)
    w[np.arange(wl.C), perm] = 1.0
    assert np.array_equal(run_fused(wl, w), plain[:, perm])


def test_fused_workspace_also_serves_the_plain_calls(oracle):
    wl = wk.make_random(743, 2, 6, 40, 72, 4, 13, x_mean=0.4)
    w_fuse, b_fuse, lkc = pointwise_weights(744, wl.C, wl.Ca)
    x = gu.to_dev_x(wl.x, wl.dtype)
    ws = binding.new_fused_workspace(wl.N, wl.Ca, wl.H, wl.W, x.dtype, True)
    want_plain = gu.run_forward(wl)
    want_fused = run_fused(wl, w_fuse, b_fuse, lkc)
    for _ in range(2):
        out = binding.convattn_fused_forward(x, wl.Ca, gu.dev(wl.lk), gu.dev(w_fuse), ws, b_fuse=gu.dev(b_fuse),
                                             lk_c=gu.dev(lkc), gen=gu.gen_params(wl))
        assert np.array_equal(out.cpu().numpy(), want_fused)
        assert np.array_equal(gu.run_forward(wl, ws=ws), want_plain)
    assert binding.workspace_errors(ws) == 0


# ------------------------------------------------------------------ benchmark shapes at full size

@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_fused_benchmark_workloads_full_size(oracle, idx):
    wl = wk.make_config(idx)
    w_fuse, b_fuse, lkc = pointwise_weights(750 + idx, wl.C, wl.Ca)
    check_fused(wl, oracle, w_fuse, b_fuse, None, None)
    if idx in (1, 3):
        check_fused(wl, oracle, w_fuse, b_fuse, lkc, residual_for(wl, 760 + idx))


def test_fused_large_model_shape(oracle):
    # C = 192, 48 attention channels, two-layer estimator: three passes of 64 output channels
    wl = wk.make_random(770, 1, 192, 90, 160, 48, 13, hidden=24, bias=True, x_mean=0.25)
    w_fuse, b_fuse, lkc = pointwise_weights(771, wl.C, wl.Ca)
    check_fused(wl, oracle, w_fuse, b_fuse, lkc, residual_for(wl, 772))
