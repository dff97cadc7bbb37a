"""Helpers shared by the GPU parity tests: move a Workload to the device, run the
HIP path through the C ABI, and compare with the CPU oracle."""
import numpy as np
import torch

from paper_2503_06671_amd import binding, workloads as wk

TOL = {wk.F32: 1e-5, wk.BF16: 2e-2}


def to_dev_x(x_np, dtype):
    if dtype == wk.F32:
        return torch.from_numpy(x_np).cuda()
    return torch.from_numpy(x_np.view(np.int16)).cuda().view(torch.bfloat16)


def out_to_np(out, dtype):
    if dtype == wk.F32:
        return out.cpu().numpy()
    return out.view(torch.int16).cpu().numpy().view(np.uint16)


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def gen_params(wl):
    return binding.GenParams(dev(wl.w_up), dev(wl.b_up), wl.hidden, dev(wl.w_down), dev(wl.b_down))


def run_forward(wl, use_gen=True, dk_in=None, lk=None, ws=None):
    """Full forward on the GPU (in a fresh workspace unless one is given).  Returns out as
    numpy in the storage dtype."""
    x = to_dev_x(wl.x, wl.dtype)
    lk_d = dev(wl.lk if lk is None else lk)
    if ws is None:
        ws = binding.new_workspace(wl.N, wl.Ca, wl.H, wl.W)
    gen = gen_params(wl) if use_gen else None
    dk_d = dev(dk_in) if dk_in is not None else None
    out = torch.full_like(x, float("nan"))
    binding.convattn_forward(x, wl.Ca, lk_d, ws, gen=gen, dk_in=dk_d, out=out)
    assert binding.workspace_errors(ws) == 0
    torch.cuda.synchronize()
    return out_to_np(out, wl.dtype)


def run_dk(wl, ws=None):
    x = to_dev_x(wl.x, wl.dtype)
    if ws is None:
        ws = binding.new_workspace(wl.N, wl.Ca, wl.H, wl.W)
    dk = binding.dynkernel_gen(x, wl.Ca, gen_params(wl), ws)
    assert binding.workspace_errors(ws) == 0
    return dk.cpu().numpy()


def att_as_f64(out_np, wl):
    a = out_np[:, :wl.Ca]
    if wl.dtype == wk.BF16:
        a = wk.bf16_bits_to_f32(a)
    return a.astype(np.float64)


def assert_att_close(got_att, ref_att, dtype, what=""):
    """Normwise max|d|/max|ref| <= tol, and elementwise |d| <= tol*(|ref| + rms(ref))."""
    tol = TOL[dtype]
    if ref_att.size == 0:
        return 0.0
    assert np.isfinite(got_att).all(), f"{what}: non-finite output"
    d = np.abs(got_att - ref_att)
    scale = np.abs(ref_att).max()
    rms = float(np.sqrt(np.mean(ref_att ** 2)))
    if scale == 0:
        assert d.max() == 0, what
        return 0.0
    rel = d.max() / scale
    assert rel <= tol, f"{what}: normwise error {rel:.3e} > {tol}"
    bad = d > tol * (np.abs(ref_att) + rms)
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond the elementwise bound"
    return rel


def assert_identity_bits(out_np, wl, what=""):
    assert np.array_equal(out_np[:, wl.Ca:].view(np.uint8), wl.x[:, wl.Ca:].view(np.uint8)), \
        f"{what}: pass-through channels differ"


def assert_dk_close(dk_gpu, dk_ref, what=""):
    if dk_ref.size == 0:
        return
    scale = np.abs(dk_ref).max()
    d = np.abs(dk_gpu.astype(np.float64) - dk_ref).max()
    if scale == 0:
        assert d == 0
    else:
        assert d / scale <= 1e-5, f"{what}: dk error {d / scale:.3e}"
