"""GPU parity of esc_convattn_backward (gradients of the depth-wise ConvAttn forward,
Eq. 4 lines 1-4 without Conv_fuse) against the CPU oracle, through the C ABI.

Bars (normwise max|d| / max|ref| per tensor, plus the elementwise bound of
gpu_util.assert_att_close for grad_x): grad_x within 1e-5 (fp32 storage) / 2e-2 (bf16
storage: one or two roundings to bf16 at the store); identity channels of grad_x are
bit copies of grad_out; the fp32 parameter gradients (grad_lk, grad_dk, estimator) within
5e-5 in both modes - they are sums of up to N*H*W fp32 products (relative rounding error
of a blocked sum ~ sqrt(terms) * 2^-24 against a result of size ~ sqrt(terms)), then a few
hundred more multiply-adds through the estimator."""
import numpy as np
import pytest
import torch

from paper_2503_06671_amd import binding, workloads as wk
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu

F32, BF16 = wk.F32, wk.BF16
PARAM_TOL = 5e-5


def grad_out_for(wl, seed):
    go = np.random.default_rng(seed).standard_normal(wl.x.shape).astype(np.float32)
    return wk.f32_to_bf16_bits(go) if wl.dtype == BF16 else go


def close(got, ref, tol, what):
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    if ref.size == 0:
        return
    scale = np.abs(ref).max()
    d = np.abs(got - ref).max()
    assert np.isfinite(got).all(), what
    assert d <= tol * scale if scale > 0 else d == 0, f"{what}: {d / max(scale, 1e-300):.3e} > {tol}"


def run_backward(wl, go, use_gen=True, dk_in=None, lk=None, accumulate=False, grads=None):
    x, g = gu.to_dev_x(wl.x, wl.dtype), gu.to_dev_x(go, wl.dtype)
    ws = binding.new_backward_workspace(wl.N, wl.Ca, wl.H, wl.W, wl.Ks, wl.hidden if use_gen else 0)
    res = binding.convattn_backward(x, g, wl.Ca, gu.dev(wl.lk if lk is None else lk), ws,
                                    gen=gu.gen_params(wl) if use_gen and wl.Ca > 0 else None, dk_in=gu.dev(dk_in),
                                    accumulate=accumulate, grads=grads)
    assert binding.workspace_errors(ws) == 0
    torch.cuda.synchronize()
    return res


def check_backward(wl, oracle, seed, what=None):
    what = what or f"backward {wl.name}"
    print(f"[case] {what}", flush=True)
    go = grad_out_for(wl, seed)
    ref = oracle.convattn_backward(wl.x, go, wl.Ca, wl.lk, wl.dtype, hidden=wl.hidden, w_up=wl.w_up, b_up=wl.b_up,
                                   w_down=wl.w_down, b_down=wl.b_down)
    got = run_backward(wl, go)
    gx = gu.out_to_np(got["grad_x"], wl.dtype)
    assert np.array_equal(gx[:, wl.Ca:], go[:, wl.Ca:]), f"{what}: identity channels of grad_x differ from grad_out"
    gx_att = (wk.bf16_bits_to_f32(gx[:, :wl.Ca]) if wl.dtype == BF16 else gx[:, :wl.Ca]).astype(np.float64)
    gu.assert_att_close(gx_att, ref["dx"][:, :wl.Ca], wl.dtype, what + " grad_x")
    close(got["grad_lk"].cpu().numpy(), ref["dlk"], PARAM_TOL, what + " grad_lk")
    close(got["grad_dk"].cpu().numpy(), ref["ddk"], PARAM_TOL, what + " grad_dk")
    for name, key in (("grad_w_up", "dw_up"), ("grad_b_up", "db_up"), ("grad_w_down", "dw_down"), ("grad_b_down", "db_down")):
        if name in got:
            close(got[name].cpu().numpy(), ref[key], PARAM_TOL, what + " " + name)
    return got, ref


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("Ks", list(range(1, 32, 2)))
def test_backward_every_kernel_size(oracle, dtype, Ks):
    # two column tiles and two row tiles of the correlation kernel with ragged tails
    wl = wk.make_random(1100 + Ks, 2, 5, 41, 75, 3, Ks, dtype=dtype, x_mean=0.4)
    check_backward(wl, oracle, 1101 + Ks)


@pytest.mark.parametrize("Ks", [1, 3, 5, 7, 9, 11, 13, 15, 17])
def test_backward_bf16_rows_of_whole_pieces(oracle, Ks):
    # bf16 storage, W % 8 == 0: the correlation on the matrix cores (windows up to 15 x 15) fetches
    # its tiles in 16-byte pieces - three column tiles, two row tiles, ragged at both edges
    wl = wk.make_random(1150 + Ks, 2, 6, 45, 136, 4, Ks, dtype=BF16, x_mean=0.4)
    check_backward(wl, oracle, 1151 + Ks)


@pytest.mark.parametrize("N,C,H,W,Ca,Ks,hidden,bias,dtype", [
    (2, 20, 40, 72, 16, 13, 8, True, F32),     # the paper's estimator (two layers, GELU)
    (3, 8, 9, 11, 4, 5, 4, False, BF16),       # odd planes
    (1, 50, 20, 24, 48, 7, 24, True, F32),     # the larger model's slice
    (1, 5, 1, 1, 2, 3, 0, True, F32),          # a single pixel
    (40, 6, 12, 12, 4, 3, 0, False, F32),      # many small images: sums over the batch
    (1, 4, 70, 200, 4, 9, 0, False, BF16),     # no identity channels, several tiles
])
def test_backward_shapes_and_estimators(oracle, N, C, H, W, Ca, Ks, hidden, bias, dtype):
    wl = wk.make_random(1200 + H + Ca, N, C, H, W, Ca, Ks, dtype=dtype, hidden=hidden, bias=bias, x_mean=0.4)
    check_backward(wl, oracle, 1201)


def test_backward_with_given_dk_shared_filter_and_no_attention_channels(oracle):
    wl = wk.make_random(1300, 2, 6, 30, 70, 4, 13, x_mean=0.3)
    go = grad_out_for(wl, 1301)
    dk = np.random.default_rng(1302).standard_normal((2, 4, 3, 3)).astype(np.float32)
    ref = oracle.convattn_backward(wl.x, go, 4, wl.lk, dk_in=dk)
    got = run_backward(wl, go, use_gen=False, dk_in=dk)
    gu.assert_att_close(got["grad_x"].cpu().numpy()[:, :4].astype(np.float64), ref["dx"][:, :4], F32, "given dk")
    close(got["grad_dk"].cpu().numpy(), ref["ddk"], PARAM_TOL, "given dk: grad_dk")
    # one filter shared by all channels: its gradient sums over the channels
    shared = wl.lk[2].copy()
    ref = oracle.convattn_backward(wl.x, go, 4, shared, w_up=wl.w_up)
    got = run_backward(wl, go, lk=shared)
    assert tuple(got["grad_lk"].shape) == (13, 13)
    close(got["grad_lk"].cpu().numpy(), ref["dlk"], PARAM_TOL, "shared filter grad_lk")
    gu.assert_att_close(got["grad_x"].cpu().numpy()[:, :4].astype(np.float64), ref["dx"][:, :4], F32, "shared filter")
    # C_a = 0: grad_x is grad_out
    wl0 = wk.make_random(1303, 2, 5, 17, 19, 0, 5)
    go0 = grad_out_for(wl0, 1304)
    got = run_backward(wl0, go0, use_gen=False)
    assert np.array_equal(got["grad_x"].cpu().numpy(), go0)


def test_backward_accumulates_parameter_gradients_when_asked(oracle):
    # two modules sharing one LK (and, here, one estimator): the second call adds to the first's gradients
    a = wk.make_random(1400, 2, 6, 24, 40, 4, 5, hidden=4, bias=True, x_mean=0.3)
    b = wk.make_random(1401, 2, 6, 24, 40, 4, 5, hidden=4, bias=True, x_mean=-0.2)
    b.lk, b.w_up, b.b_up, b.w_down, b.b_down = a.lk, a.w_up, a.b_up, a.w_down, a.b_down
    go_a, go_b = grad_out_for(a, 1402), grad_out_for(b, 1403)
    first = run_backward(a, go_a)
    keep = {k: v for k, v in first.items() if k not in ("grad_x", "grad_dk")}
    second = run_backward(b, go_b, accumulate=True, grads=keep)
    ra = oracle.convattn_backward(a.x, go_a, 4, a.lk, hidden=4, w_up=a.w_up, b_up=a.b_up, w_down=a.w_down, b_down=a.b_down)
    rb = oracle.convattn_backward(b.x, go_b, 4, b.lk, hidden=4, w_up=b.w_up, b_up=b.b_up, w_down=b.w_down, b_down=b.b_down)
    for name, key in (("grad_lk", "dlk"), ("grad_w_up", "dw_up"), ("grad_b_up", "db_up"), ("grad_w_down", "dw_down"),
                      ("grad_b_down", "db_down")):
        close(second[name].cpu().numpy(), ra[key] + rb[key], PARAM_TOL, "accumulated " + name)


def test_delta_kernel_backward_is_exact():
    # LK = centre delta, DK = 0: the forward is the identity, so grad_x equals grad_out bit for bit
    wl = wk.make_random(1500, 2, 5, 50, 90, 3, 13)
    lk = np.zeros((3, 13, 13), np.float32)
    lk[:, 6, 6] = 1.0
    go = grad_out_for(wl, 1501)
    got = run_backward(wl, go, use_gen=False, lk=lk)
    assert np.array_equal(got["grad_x"].cpu().numpy(), go)


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_backward_benchmark_workloads_full_size(oracle, idx):
    wl = wk.make_config(idx)
    check_backward(wl, oracle, 1600 + idx)


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_backward_and_dense_calls_replay_from_a_captured_graph(dtype):
    # The multi-launch calls captured into one graph: replays, with plain calls and
    # synchronisations in between, must reproduce the plain calls bit for bit (every sum has a
    # fixed order; nothing in the workspace may carry over from one call to the next).
    wl = wk.make_random(1400, 3, 8, 45, 136, 4, 13, dtype=dtype, hidden=4, bias=True, x_mean=0.4)
    go = grad_out_for(wl, 1401)
    x, g = gu.to_dev_x(wl.x, wl.dtype), gu.to_dev_x(go, wl.dtype)
    lk, gen = gu.dev(wl.lk), gu.gen_params(wl)
    lkd = gu.dev((np.random.default_rng(1402).standard_normal((4, 4, 13, 13)) / 26.0).astype(np.float32))
    ws_b = binding.new_backward_workspace(wl.N, wl.Ca, wl.H, wl.W, wl.Ks, wl.hidden)
    ws_d = binding.new_dense_workspace(wl.N, wl.Ca, wl.H, wl.W, 13)
    stream = torch.cuda.Stream()

    def fresh():
        w_down, b_down, w_up, b_up = gen.tensors
        return {"grad_x": torch.full_like(x, float("nan")), "grad_lk": torch.full_like(lk, float("nan")),
                "grad_dk": torch.full((wl.N, wl.Ca, 3, 3), float("nan"), device="cuda"),
                "grad_w_up": torch.full_like(w_up, float("nan")), "grad_b_up": torch.full_like(b_up, float("nan")),
                "grad_w_down": torch.full_like(w_down, float("nan")), "grad_b_down": torch.full_like(b_down, float("nan"))}

    def enqueue(grads, out_d):
        binding.convattn_backward(x, g, wl.Ca, lk, ws_b, gen=gen, grads=grads, stream=stream)
        binding.convattn_dense_forward(x, wl.Ca, lkd, ws_d, gen=gen, out=out_d, stream=stream)

    want, want_d = fresh(), torch.full_like(x, float("nan"))
    with torch.cuda.stream(stream):
        enqueue(want, want_d)
    torch.cuda.synchronize()
    got, got_d = fresh(), torch.full_like(x, float("nan"))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        enqueue(got, got_d)
    scratch, scratch_d = fresh(), torch.empty_like(x)
    for rep in range(3):
        for t in list(got.values()) + [got_d]:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        assert binding.workspace_errors(ws_b, stream) == 0 and binding.workspace_errors(ws_d, stream) == 0
        print(f"[case] backward + dense graph replay {rep}, {wl.name}", flush=True)
        for k in want:
            assert torch.equal(got[k].view(torch.uint8), want[k].view(torch.uint8)), k
        assert torch.equal(got_d.view(torch.uint8), want_d.view(torch.uint8))
        with torch.cuda.stream(stream):  # plain work on the same workspaces between replays
            enqueue(scratch, scratch_d)
        torch.cuda.synchronize()
