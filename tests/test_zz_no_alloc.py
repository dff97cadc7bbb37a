"""The entry point that allocates nothing (esc_convattn_forward_noalloc): its output must
equal esc_convattn_forward's bit for bit - same checks, same plan, same kernel; only the
mailboxes live in the library's own scratch array - on calls in a row that share that
array, the later ones with smaller inputs, and it must refuse shapes beyond the scratch."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2503_06671_amd import binding, workloads as wk
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def run_pair(wl, oracle):
    print(f"[case] no-alloc entry point, {wl.name}", flush=True)
    x = gu.to_dev_x(wl.x, wl.dtype)
    lk, gen = gu.dev(wl.lk), gu.gen_params(wl)
    want = torch.full_like(x, float("nan"))
    ws = binding.new_workspace(wl.N, wl.Ca, wl.H, wl.W)
    binding.convattn_forward(x, wl.Ca, lk, ws, gen=gen, out=want)
    assert binding.workspace_errors(ws) == 0
    got = torch.full_like(x, float("nan"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.convattn_forward(x, wl.Ca, lk, None, gen=gen, out=got)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    got_np, want_np = gu.out_to_np(got, wl.dtype), gu.out_to_np(want, wl.dtype)
    assert np.array_equal(got_np.view(np.uint8), want_np.view(np.uint8)), "differs from esc_convattn_forward"
    # and, like every other path, against the oracle
    ref_att, _, _ = oracle.forward_workload(wl, want_out=False)
    gu.assert_identity_bits(got_np, wl, wl.name)
    gu.assert_att_close(gu.att_as_f64(got_np, wl), ref_att, wl.dtype, wl.name)


def test_noalloc_entry_point_matches_the_workspace_one_on_calls_in_a_row(oracle):
    # a larger call first, then smaller ones of other shapes, kinds and storage types, then
    # the first again: all share the device's one scratch array
    cases = [
        wk.make_config(1),                                                        # 180 x 320, fused pooling, gen hop
        wk.make_random(901, 2, 6, 40, 72, 4, 13, dtype=wk.BF16, x_mean=0.4),      # smaller, bf16
        wk.make_random(902, 40, 6, 30, 30, 4, 3, dtype=wk.F32, x_mean=0.4),       # many small images, direct form
        wk.make_random(903, 1, 10, 200, 704, 8, 7, dtype=wk.F32, hidden=4, x_mean=0.4),  # channel means, queue-dealt
        wk.make_random(904, 1, 3, 5, 7, 2, 5, dtype=wk.F32, x_mean=0.4),          # tiny
        wk.make_config(1),
    ]
    for wl in cases:
        run_pair(wl, oracle)


def test_noalloc_entry_point_refuses_shapes_beyond_its_scratch():
    # 4096 images of 64 channels need more mailboxes than the built-in scratch holds: refused
    # on the host, before anything is looked up or launched (fake pointers)
    lib = binding.load_library()
    N, Ca, H, W = 4096, 64, 8, 8
    assert binding.workspace_bytes(N, Ca, H, W) > binding.NOALLOC_SCRATCH_BYTES
    st = lib.esc_convattn_forward_noalloc(0x10000, 0, N, Ca, H, W, Ca, 0x9000000, 3, 9, None, None, 0x20000000, None)
    assert st == 5 and "scratch" in binding.status_string(st)
