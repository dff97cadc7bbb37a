"""GPU parity of esc_convattn_dense_forward (the module with the dense large kernel of the
paper's main variants, Sec. 3 / Eq. 4 line 3) against the CPU oracle, through the C ABI.
Bars as for the depth-wise forward: attention slice within 1e-5 (fp32 storage) / 2e-2 (bf16
storage) of the oracle's unrounded float64 result, normwise and elementwise; identity
channels bit-exact."""
import numpy as np
import pytest
import torch

from paper_2503_06671_amd import binding, workloads as wk
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

F32, BF16 = wk.F32, wk.BF16


def dense_kernel(seed, Ca, Ks):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((Ca, Ca, Ks, Ks)) / (Ks * np.sqrt(max(Ca, 1)))).astype(np.float32)


def run_dense(wl, lk, use_gen=True, dk_in=None):
    x = gu.to_dev_x(wl.x, wl.dtype)
    ws = binding.new_dense_workspace(wl.N, wl.Ca, wl.H, wl.W, lk.shape[2])
    out = torch.full_like(x, float("nan"))
    binding.convattn_dense_forward(x, wl.Ca, gu.dev(lk), ws, gen=gu.gen_params(wl) if use_gen and wl.Ca > 0 else None,
                                   dk_in=gu.dev(dk_in), out=out)
    assert binding.workspace_errors(ws) == 0
    torch.cuda.synchronize()
    return gu.out_to_np(out, wl.dtype)


def check_dense(wl, lk, oracle, what=None):
    what = what or f"dense {wl.name}"
    print(f"[case] {what}", flush=True)
    ref, _, _ = oracle.convattn_dense_forward(wl.x, wl.Ca, lk, wl.dtype, hidden=wl.hidden, w_up=wl.w_up, b_up=wl.b_up,
                                              w_down=wl.w_down, b_down=wl.b_down, want_out=False)
    got = run_dense(wl, lk)
    gu.assert_identity_bits(got, wl, what)
    return gu.assert_att_close(gu.att_as_f64(got, wl), ref, wl.dtype, what)


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("N,C,H,W,Ca,Ks", [
    (2, 20, 21, 45, 16, 13),   # the paper's shape of LK on ragged tiles
    (1, 6, 9, 11, 3, 5),       # fewer channels than a tile of 16, odd plane (element-wise copy)
    (2, 24, 17, 40, 20, 3),    # two chunks of input channels, two tiles of output channels
    (1, 50, 10, 33, 48, 7),    # three chunks (the larger model's slice)
    (1, 70, 9, 20, 64, 3),     # four chunks
    (3, 5, 8, 8, 2, 1),        # a 1 x 1 dense kernel (embedded in 3 x 3)
    (1, 18, 30, 70, 16, 17),   # the largest dense kernel
    (1, 4, 1, 1, 4, 9),        # a single pixel, no identity channels
    (30, 18, 12, 20, 16, 5),   # many small images
])
def test_dense_small_shapes(oracle, dtype, N, C, H, W, Ca, Ks):
    wl = wk.make_random(900 + C + H, N, C, H, W, Ca, Ks, dtype=dtype, x_mean=0.3)
    check_dense(wl, dense_kernel(901 + Ca, Ca, Ks), oracle)


def test_dense_two_layer_estimator_given_dk_and_no_dk(oracle):
    wl = wk.make_random(910, 2, 20, 24, 40, 16, 9, hidden=8, bias=True, x_mean=0.5)
    lk = dense_kernel(911, 16, 9)
    check_dense(wl, lk, oracle)
    dk = np.random.default_rng(912).standard_normal((2, 16, 3, 3)).astype(np.float32)
    ref, _, _ = oracle.convattn_dense_forward(wl.x, wl.Ca, lk, dk_in=dk, want_out=False)
    gu.assert_att_close(gu.att_as_f64(run_dense(wl, lk, use_gen=False, dk_in=dk), wl), ref, F32, "given dk")
    ref, _, _ = oracle.convattn_dense_forward(wl.x, wl.Ca, lk, want_out=False)
    gu.assert_att_close(gu.att_as_f64(run_dense(wl, lk, use_gen=False), wl), ref, F32, "no dk")


def test_single_entry_dense_kernel_is_an_exact_shift():
    # lk[co=2, ci=1, 1, 3] = 1, Ks = 5: out[2][y,x] = x[1][y-1, x+1] exactly, zero in other channels
    wl = wk.make_random(913, 1, 6, 20, 50, 4, 5)
    lk = np.zeros((4, 4, 5, 5), np.float32)
    lk[2, 1, 1, 3] = 1.0
    got = run_dense(wl, lk, use_gen=False)
    want = np.zeros((20, 50), np.float32)
    want[1:, :-1] = wl.x[0, 1, :-1, 1:]
    assert np.array_equal(got[0, 2], want)
    assert not got[0, [0, 1, 3]].any()
    assert np.array_equal(got[:, 4:], wl.x[:, 4:])


def test_no_attention_channels_is_a_pure_copy():
    wl = wk.make_random(914, 2, 5, 17, 19, 0, 5)
    got = run_dense(wl, np.zeros((0, 0, 5, 5), np.float32), use_gen=False)
    assert np.array_equal(got.view(np.uint8), wl.x.view(np.uint8))


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_dense_base_pointers_off_the_vector_alignment(oracle, dtype):
    # W % 8 == 0, but x and out start one element past a 16-byte boundary (views into larger
    # buffers): the tile fetch and the pass-through copy must take their element-wise forms,
    # and nothing outside the view may be written.  Then the aligned call on the same data (the
    # 16-byte tile fetch of the bf16 matrix path) must give the same attention slice bit for bit.
    wl = wk.make_random(940, 2, 19, 21, 72, 16, 7, dtype=dtype, x_mean=0.4)
    lk = dense_kernel(941, 16, 7)
    print(f"[case] dense, unaligned base, {wl.name}", flush=True)
    ref, _, _ = oracle.convattn_dense_forward(wl.x, wl.Ca, lk, wl.dtype, hidden=wl.hidden, w_up=wl.w_up, b_up=wl.b_up,
                                              w_down=wl.w_down, b_down=wl.b_down, want_out=False)
    aligned = run_dense(wl, lk)
    x_al = gu.to_dev_x(wl.x, wl.dtype)
    numel = x_al.numel()
    for x_shift, out_shift in ((1, 1), (1, 0), (0, 3)):
        xb = torch.zeros(numel + 8, dtype=x_al.dtype, device="cuda")
        ob = torch.full((numel + 8,), float("nan"), dtype=x_al.dtype, device="cuda")
        x = xb[x_shift:x_shift + numel].view(x_al.shape)
        x.copy_(x_al)
        out = ob[out_shift:out_shift + numel].view(x_al.shape)
        ws = binding.new_dense_workspace(wl.N, wl.Ca, wl.H, wl.W, 7)
        binding.convattn_dense_forward(x, wl.Ca, gu.dev(lk), ws, gen=gu.gen_params(wl), out=out)
        assert binding.workspace_errors(ws) == 0
        got = gu.out_to_np(out, wl.dtype)
        gu.assert_identity_bits(got, wl, "dense, unaligned base")
        gu.assert_att_close(gu.att_as_f64(got, wl), ref, wl.dtype, "dense, unaligned base")
        assert np.array_equal(got.view(np.uint8), aligned.view(np.uint8))
        edge = ob.view(torch.int16 if dtype == BF16 else torch.int32)
        nan_bits = torch.full((1,), float("nan"), dtype=x_al.dtype).view(edge.dtype).item()
        assert all(int(v) == nan_bits for v in edge[:out_shift].tolist() + edge[out_shift + numel:].tolist())


@pytest.mark.parametrize("Ks", [1, 3, 5, 7, 9, 11, 15, 17])
def test_dense_bf16_matrix_path_every_kernel_size_on_eight_row_tiles(oracle, Ks):
    # bf16 storage with 16 channels runs one compiled kernel per kernel size and tile height:
    # 44 images of 43 x 64 give 8-row tiles (enough blocks to fill the chip twice), ragged at the
    # bottom edge; the small shapes above take the 4-row tiles, the benchmark shapes Ks = 13.
    wl = wk.make_random(950 + Ks, 44, 17, 43, 64, 16, Ks, dtype=BF16, x_mean=0.2)
    check_dense(wl, dense_kernel(951 + Ks, 16, Ks), oracle)


@pytest.mark.parametrize("W", [72, 45])
@pytest.mark.parametrize("Ks", [1, 3, 5, 7, 9, 11, 13, 15])
def test_dense_fp32_on_bf16_terms_every_kernel_size(oracle, Ks, W):
    # fp32 storage with up to 16 channels and Ks <= 13 runs the bf16 matrix instructions on three
    # exact terms per value and weight (Ks = 15 stays on the fp32 instructions); W = 72 takes the
    # 16-byte tile fetch, W = 45 the element-wise one; fewer channels than 16, ragged tiles.
    wl = wk.make_random(960 + Ks + W, 2, 14, 21, W, 12, Ks, dtype=F32, x_mean=0.2)
    rel = check_dense(wl, dense_kernel(961 + Ks, 12, Ks), oracle)
    assert rel <= 2e-6, rel  # (six of the nine products of terms: fp32 accuracy, far inside the 1e-5 bar)


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_dense_benchmark_shapes_full_size(oracle, idx):
    wl = wk.make_config(idx)
    check_dense(wl, dense_kernel(920 + idx, wl.Ca, 13), oracle)
