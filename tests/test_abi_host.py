"""Host-only checks of the C ABI: the library loads, exports what the header
declares, and rejects bad arguments before anything is launched (so these run
without a GPU)."""
import ctypes
import os
import re

import numpy as np

import pytest

from paper_2503_06671_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

OK, E_NULL, E_SHAPE, E_DTYPE, E_UNSUP, E_WS, E_ALIAS, E_HIP = range(8)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2503_06671_amd import build
        build.build()
    return binding.load_library()


def header_functions():
    text = open(os.path.join(ROOT, "include", "esc_convattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(esc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = header_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    seen = {binding.status_string(s) for s in range(8)}
    assert len(seen) == 8 and binding.status_string(0) == "ok"
    assert binding.status_string(99) == "unknown status"


def test_workspace_bytes(lib):
    a = lib.esc_workspace_bytes(1, 16, 180, 320)
    assert a > 0 and a % 256 == 0
    assert lib.esc_workspace_bytes(64, 16, 64, 64) > lib.esc_workspace_bytes(1, 16, 64, 64)
    assert lib.esc_workspace_bytes(1, 16, 540, 960) >= a
    assert lib.esc_workspace_bytes(0, 16, 8, 8) == 0
    assert lib.esc_workspace_bytes(1, -1, 8, 8) == 0
    assert lib.esc_workspace_bytes(1, 16, 0, 8) == 0
    assert lib.esc_workspace_bytes(1, 16, 65536, 65536) == 0
    assert lib.esc_workspace_bytes(1, 0, 8, 8) >= 256


def fwd(lib, x=0x10000, dt=0, N=1, C=64, H=8, W=8, Ca=16, lk=0x20000, Ks=13, stride=169, gen=None,
        dk=None, out=0x90000, ws=0x30000 * 256, ws_bytes=1 << 20):
    return lib.esc_convattn_forward(x, dt, N, C, H, W, Ca, lk, Ks, stride, gen, dk, out, ws, ws_bytes, None)


def gen_struct(hidden=0, w_down=None, b_down=None, w_up=0x40000, b_up=None):
    return ctypes.byref(binding._GenParams(hidden, w_down, b_down, w_up, b_up))


def test_forward_rejects_bad_arguments_before_launch(lib):
    # the device "pointers" are fake: every call below must fail in validation
    assert fwd(lib, x=None) == E_NULL
    assert fwd(lib, out=None) == E_NULL
    assert fwd(lib, lk=None) == E_NULL
    assert fwd(lib, dt=2) == E_DTYPE
    assert fwd(lib, N=0) == E_SHAPE
    assert fwd(lib, H=0) == E_SHAPE
    assert fwd(lib, Ca=65) == E_SHAPE
    assert fwd(lib, Ca=-1) == E_SHAPE
    assert fwd(lib, Ks=0) == E_SHAPE
    assert fwd(lib, Ks=12) == E_UNSUP
    assert fwd(lib, Ks=33) == E_UNSUP
    assert fwd(lib, stride=100) == E_SHAPE
    assert fwd(lib, C=512, Ca=300) == E_UNSUP
    assert fwd(lib, H=65536, W=65536) == E_UNSUP
    assert fwd(lib, out=0x10000 + 4 * 64 * 64 - 4) == E_ALIAS      # last element of x
    assert fwd(lib, out=0x10000) == E_ALIAS
    assert fwd(lib, x=0x10002) == E_SHAPE                           # misaligned for fp32
    assert fwd(lib, ws=None) == E_WS
    assert fwd(lib, gen=gen_struct(), ws=None) == E_WS
    assert fwd(lib, gen=gen_struct(), ws=0x30000 * 256 + 8) == E_WS
    assert fwd(lib, gen=gen_struct(), ws_bytes=16) == E_WS
    assert fwd(lib, gen=gen_struct(w_up=None)) == E_NULL
    assert fwd(lib, gen=gen_struct(hidden=8, w_down=None)) == E_NULL
    assert fwd(lib, gen=gen_struct(hidden=-1)) == E_SHAPE
    assert fwd(lib, gen=gen_struct(hidden=1000, w_down=0x50000)) == E_UNSUP


def test_dynkernel_gen_rejects_bad_arguments_before_launch(lib):
    def gen(x=0x10000, dt=0, N=1, C=64, H=8, W=8, Ca=16, g=gen_struct(), dk=0x60000, ws=0x30000 * 256,
            ws_bytes=1 << 20):
        return lib.esc_dynkernel_gen(x, dt, N, C, H, W, Ca, g, dk, ws, ws_bytes, None)
    assert gen(x=None) == E_NULL
    assert gen(g=None) == E_NULL
    assert gen(dk=None) == E_NULL
    assert gen(dt=7) == E_DTYPE
    assert gen(W=-3) == E_SHAPE
    assert gen(ws=None) == E_WS
    assert gen(ws_bytes=0) == E_WS
    assert gen(Ca=0) == OK          # nothing to do, nothing launched
    assert lib.esc_workspace_init(None, 1024, None) == E_WS
    assert lib.esc_workspace_init(0x1001, 1024, None) == E_WS


def test_noalloc_entry_point_validates_before_anything_else(lib):
    def na(x=0x10000, dt=0, N=1, C=64, H=8, W=8, Ca=16, lk=0x20000, Ks=13, stride=169, gen=None, dk=None,
           out=0x90000):
        return lib.esc_convattn_forward_noalloc(x, dt, N, C, H, W, Ca, lk, Ks, stride, gen, dk, out, None)
    assert na(x=None) == E_NULL
    assert na(out=None) == E_NULL
    assert na(Ks=12) == E_UNSUP
    assert na(N=0) == E_SHAPE
    assert na(out=0x10000) == E_ALIAS
    # a shape whose mailboxes do not fit the built-in scratch is refused as a workspace error
    assert lib.esc_workspace_bytes(4096, 64, 8, 8) > binding.NOALLOC_SCRATCH_BYTES
    assert na(N=4096, Ca=64, out=0x20000000) == E_WS
    text = open(os.path.join(ROOT, "include", "esc_convattn.h")).read()
    assert re.search(r"#define\s+ESC_NOALLOC_SCRATCH_BYTES\s+\(1u << 20\)", text)


def test_fused_forward_rejects_bad_arguments_before_launch(lib):
    def fu(x=0x10000, dt=0, N=1, C=64, H=8, W=8, Ca=16, lkc=None, lk=0x20000, Ks=13, stride=169, gen=None, dk=None,
           wf=0x50000, bf=None, res=None, out=0x90000, ws=0x30000 * 256, ws_bytes=1 << 22):
        return lib.esc_convattn_fused_forward(x, dt, N, C, H, W, Ca, lkc, lk, Ks, stride, gen, dk, wf, bf, res, out,
                                              ws, ws_bytes, None)
    assert fu(x=None) == E_NULL
    assert fu(out=None) == E_NULL
    assert fu(wf=None) == E_NULL
    assert fu(lk=None) == E_NULL
    assert fu(dt=3) == E_DTYPE
    assert fu(Ks=4) == E_UNSUP
    assert fu(C=241, Ca=16) == E_UNSUP
    assert fu(Ca=65) == E_SHAPE
    assert fu(out=0x10000) == E_ALIAS
    assert fu(res=0x90000) == E_ALIAS                     # residual overlaps out
    assert fu(res=0x90002) == E_SHAPE                     # misaligned residual
    assert fu(ws=None) == E_WS
    # the fused call needs room for F_res (and F_pw, DK with LK^c) behind the forward's workspace
    plain = lib.esc_workspace_bytes(1, 16, 8, 8)
    need = lib.esc_fused_workspace_bytes(1, 16, 8, 8, 0, 0)
    need_c = lib.esc_fused_workspace_bytes(1, 16, 8, 8, 0, 1)
    assert plain < need < need_c and need % 256 == 0 and need_c % 256 == 0
    assert need - plain >= 16 * 64 * 4 and need_c - need >= 16 * 64 * 4 + 16 * 9 * 4
    assert lib.esc_fused_workspace_bytes(1, 16, 8, 8, 1, 0) < need          # bf16 slices are smaller
    assert lib.esc_fused_workspace_bytes(1, 16, 8, 8, 5, 0) == 0
    assert fu(ws_bytes=plain) == E_WS
    assert fu(ws_bytes=need, lkc=0x60000) == E_WS


def test_dense_forward_rejects_bad_arguments_before_launch(lib):
    def de(x=0x10000, dt=0, N=1, C=64, H=8, W=8, Ca=16, lk=0x20000, Ks=13, gen=None, dk=None, out=0x90000,
           ws=0x30000 * 256, ws_bytes=1 << 22):
        return lib.esc_convattn_dense_forward(x, dt, N, C, H, W, Ca, lk, Ks, gen, dk, out, ws, ws_bytes, None)
    assert de(x=None) == E_NULL
    assert de(out=None) == E_NULL
    assert de(lk=None) == E_NULL
    assert de(dt=2) == E_DTYPE
    assert de(Ks=0) == E_SHAPE
    assert de(Ks=6) == E_UNSUP
    assert de(Ks=19) == E_UNSUP                           # dense kernels stop at 17 x 17
    assert de(C=80, Ca=65) == E_UNSUP                     # and at 64 attention channels
    assert de(Ca=65) == E_SHAPE                           # C_a > C
    assert de(out=0x10000) == E_ALIAS
    assert de(out=0x90001, dt=1) == E_SHAPE               # misaligned for the storage type
    assert de(lk=0x90000 + 64) == E_ALIAS                 # weights inside out
    assert de(dk=0x90000 + 128) == E_ALIAS
    assert de(gen=gen_struct(w_up=None)) == E_NULL
    assert de(ws=None) == E_WS
    plain = lib.esc_workspace_bytes(1, 16, 8, 8)
    need = lib.esc_dense_workspace_bytes(1, 16, 8, 8, 13)
    # room for DK and for the rearranged weights behind the forward's workspace
    assert need % 256 == 0 and need - plain >= 16 * 9 * 4 + 16 * 16 * 169 * 4
    assert lib.esc_dense_workspace_bytes(1, 16, 8, 8, 3) < need
    assert lib.esc_dense_workspace_bytes(1, 16, 8, 8, 0) == 0
    assert de(ws_bytes=need - 256) == E_WS
    assert de(ws=0x90000 - 256, ws_bytes=need) == E_ALIAS  # workspace runs into out


def test_convffn_rejects_bad_arguments_before_launch(lib):
    def ff(x=0x10000, dt=0, N=1, C=64, H=8, W=8, Ch=128, w1=0x20000, b1=None, k=0x28000, bk=None, w2=0x2a000, b2=None,
           out=0x90000, ws=0x30000 * 256, ws_bytes=1 << 22):
        return lib.esc_convffn_forward(x, dt, N, C, H, W, Ch, w1, b1, k, bk, w2, b2, out, ws, ws_bytes, None)
    for name in ("x", "out", "w1", "k", "w2"):
        assert ff(**{name: None}) == E_NULL, name
    assert ff(dt=3) == E_DTYPE
    assert ff(N=0) == E_SHAPE
    assert ff(Ch=0) == E_SHAPE
    assert ff(Ch=961) == E_UNSUP                          # hidden layers up to 960 channels
    assert ff(C=241) == E_UNSUP                           # the point-wise kernel's LDS staging holds 240 channels
    assert ff(out=0x10000) == E_ALIAS
    assert ff(out=0x90002) == E_SHAPE                     # misaligned for fp32 storage
    assert ff(ws=None) == E_WS
    need = lib.esc_convffn_workspace_bytes(1, 128, 8, 8, 0)
    assert need % 256 == 0 and need >= 2 * 128 * 64 * 4   # U and V in the storage type
    assert lib.esc_convffn_workspace_bytes(1, 128, 8, 8, 1) * 2 == need
    assert lib.esc_convffn_workspace_bytes(1, 128, 8, 8, 2) == 0
    assert lib.esc_convffn_workspace_bytes(0, 128, 8, 8, 0) == 0
    assert ff(ws_bytes=need - 1) == E_WS
    assert ff(ws=0x30000 * 256 + 4, ws_bytes=need + 4) == E_WS   # not 256-byte aligned
    assert ff(ws=0x90000 - 256, ws_bytes=need) == E_ALIAS        # workspace runs into out


def test_residual_step_rejects_bad_arguments_before_launch(lib):
    def rs(f=0x10000, dt=0, N=1, C=64, H=8, W=8, Ch=128, w1=0x20000, k=0x28000, w2=0x2a000, Ca=16, lkc=None, lk=0x2c000,
           Ks=13, stride=169, gen=None, wf=0x2e000, out=0x90000, ws=0x30000 * 256, ws_bytes=1 << 22):
        return lib.esc_residual_step_forward(f, dt, N, C, H, W, Ch, w1, None, k, None, w2, None, Ca, lkc, lk, Ks, stride,
                                             gen, wf, None, out, ws, ws_bytes, None)
    for name in ("f", "out", "w1", "k", "w2", "lk", "wf"):
        assert rs(**{name: None}) == E_NULL, name
    assert rs(dt=9) == E_DTYPE
    assert rs(Ch=0) == E_SHAPE
    assert rs(Ch=961) == E_UNSUP
    assert rs(Ks=4) == E_UNSUP
    assert rs(Ks=0) == E_SHAPE
    assert rs(Ca=65) == E_SHAPE
    assert rs(stride=10) == E_SHAPE
    assert rs(out=0x10000) == E_ALIAS
    assert rs(gen=gen_struct(w_up=None)) == E_NULL
    need = lib.esc_residual_step_workspace_bytes(1, 64, 8, 8, 16, 128, 0, 0)
    fused = lib.esc_fused_workspace_bytes(1, 16, 8, 8, 0, 0)
    ffn = lib.esc_convffn_workspace_bytes(1, 128, 8, 8, 0)
    # the fused call's workspace, ConvFFN's result, ConvFFN's scratch
    assert need % 256 == 0 and need >= fused + 64 * 64 * 4 + ffn
    assert lib.esc_residual_step_workspace_bytes(1, 64, 8, 8, 16, 128, 0, 1) > need
    assert lib.esc_residual_step_workspace_bytes(1, 64, 8, 8, 65, 128, 0, 0) == 0
    assert lib.esc_residual_step_workspace_bytes(1, 64, 8, 8, 16, 0, 0, 0) == 0
    assert rs(ws=None) == E_WS
    assert rs(ws_bytes=need - 256) == E_WS
    assert rs(ws=0x90000 - 256, ws_bytes=need) == E_ALIAS


def test_backward_rejects_bad_arguments_before_launch(lib):
    def bw(x=0x10000, go=0x50000, dt=0, N=1, C=64, H=8, W=8, Ca=16, lk=0x20000, Ks=13, stride=169, gen=None, dk=None,
           gx=0x90000, glk=0x28000, ggen=None, gdk=None, acc=0, ws=0x30000 * 256, ws_bytes=1 << 22):
        return lib.esc_convattn_backward(x, go, dt, N, C, H, W, Ca, lk, Ks, stride, gen, dk, gx, glk, ggen, gdk, acc,
                                         ws, ws_bytes, None)
    assert bw(x=None) == E_NULL
    assert bw(go=None) == E_NULL
    assert bw(gx=None) == E_NULL
    assert bw(lk=None) == E_NULL
    assert bw(dt=7) == E_DTYPE
    assert bw(Ks=-1) == E_SHAPE
    assert bw(Ks=8) == E_UNSUP
    assert bw(Ks=33) == E_UNSUP
    assert bw(stride=100) == E_SHAPE                      # channel stride shorter than one kernel
    assert bw(Ca=65) == E_SHAPE
    assert bw(gx=0x10000) == E_ALIAS                      # grad_x over x
    assert bw(gx=0x50000) == E_ALIAS                      # grad_x over grad_out
    assert bw(gx=0x90002) == E_SHAPE
    assert bw(gen=gen_struct(w_up=None)) == E_NULL
    assert bw(ws=None) == E_WS
    plain = lib.esc_workspace_bytes(1, 16, 8, 8)
    need = lib.esc_backward_workspace_bytes(1, 16, 8, 8, 13, 0)
    assert need % 256 == 0 and need > plain
    assert lib.esc_backward_workspace_bytes(1, 16, 8, 8, 13, 8) >= need       # a hidden layer keeps more
    assert lib.esc_backward_workspace_bytes(1, 16, 8, 8, 13, -1) == 0
    assert lib.esc_backward_workspace_bytes(1, 16, 8, 8, 0, 0) == 0
    assert bw(ws_bytes=need - 256) == E_WS
    assert bw(ws=0x90000 - 256, ws_bytes=need) == E_ALIAS


def test_binding_refuses_cpu_tensors(lib):
    import torch
    x = torch.zeros(1, 4, 8, 8)
    with pytest.raises(TypeError):
        binding.convattn_forward(x, 2, torch.zeros(2, 3, 3), torch.zeros(1024, dtype=torch.uint8))


# ---------------------------------------------------------------- compiled kernel variants

def kernel_notes():
    """(mangled name, private segment bytes, VGPRs, static LDS bytes) of every kernel in the built
    library, read from the code objects' notes.  The library holds one offload bundle per
    translation unit."""
    import subprocess
    import tempfile
    tools = "/opt/rocm/llvm/bin"
    need = [os.path.join(tools, t) for t in ("llvm-objcopy", "clang-offload-bundler", "llvm-readelf")]
    if not all(os.path.exists(t) for t in need):
        pytest.skip("LLVM binary tools not found")
    magic = b"__CLANG_OFFLOAD_BUNDLE__"
    out = []
    with tempfile.TemporaryDirectory() as tmp:
        fat = os.path.join(tmp, "fat.bin")
        subprocess.run([need[0], f"--dump-section=.hip_fatbin={fat}", binding.LIB_PATH, os.path.join(tmp, "copy.so")],
                       check=True)
        data = open(fat, "rb").read()
        starts = []
        i = data.find(magic)
        while i >= 0:
            starts.append(i)
            i = data.find(magic, i + 1)
        for k, s in enumerate(starts):
            one, dev = os.path.join(tmp, f"b{k}.bin"), os.path.join(tmp, f"d{k}.co")
            open(one, "wb").write(data[s:starts[k + 1] if k + 1 < len(starts) else len(data)])
            subprocess.run([need[1], "--unbundle", "--type=o", f"--input={one}",
                            "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={dev}"], check=True)
            notes = subprocess.run([need[2], "--notes", dev], check=True, capture_output=True, text=True).stdout
            for block in notes.split("- .agpr_count:")[1:]:
                name = re.search(r"\.name:\s*(\S+)", block).group(1)
                scratch = int(re.search(r"\.private_segment_fixed_size:\s*(\d+)", block).group(1))
                vgprs = int(re.search(r"\.vgpr_count:\s*(\d+)", block).group(1))
                lds = int(re.search(r"\.group_segment_fixed_size:\s*(\d+)", block).group(1))
                out.append((name, scratch, vgprs, lds))
    return out


def kernel_metadata():
    """(Ks, RY, type letter, staged flavour) -> (private segment bytes, VGPRs, static LDS bytes)
    of every forward_kernel variant in the built library."""
    out = {}
    for name, scratch, vgprs, lds in kernel_notes():
        m = re.search(r"forward_kernelILi(\d+)ELi(\d+)E(\w+?)Lb([01])E", name)
        if not m:
            continue
        key = (int(m.group(1)), int(m.group(2)), "f" if m.group(3) == "f" else "b", int(m.group(4)))
        assert key not in out, key
        out[key] = (scratch, vgprs, lds)
    return out


# (Ks, RY) pairs the library is built with: both register blockings up to Ks = 17, the
# two-row one beyond, and Ks = 0 for the variant without conv items
VARIANT_SHAPES = [(0, 2)] + [(ks, ry) for ks in range(1, 32, 2) for ry in ((2, 4) if ks <= 17 else (2,))]
LDS_PER_CU = 160 * 1024


def test_kernel_variants_fit_four_blocks_per_cu_without_scratch(lib):
    # Four resident blocks per compute unit is what the grid is sized for: <= 128 VGPRs and a
    # quarter of the compute unit's LDS per block.  Any private-segment use costs every launch
    # a fixed microsecond or more: the flavour short calls use (unstaged estimator; Ks <= 13,
    # both register blockings; two-row blocks up to Ks = 15) must have none, the others next
    # to none.  Both storage types and both estimator flavours of every variant are checked.
    meta = kernel_metadata()
    want = {(ks, ry, t, st) for ks, ry in VARIANT_SHAPES for t in "fb" for st in (0, 1)}
    assert set(meta) == want, sorted(want ^ set(meta))
    for (ks, ry, t, st), (scratch, vgprs, lds) in sorted(meta.items()):
        assert vgprs <= 128, (ks, ry, t, st, vgprs)
        assert 4 * lds <= LDS_PER_CU, (ks, ry, t, st, lds)
        if st == 0 and (ks <= 13 or (ks <= 15 and ry == 2)):
            assert scratch == 0, (ks, ry, t, st, scratch)
        else:
            assert scratch <= 64, (ks, ry, t, st, scratch)


def test_dense_bf16_kernels_fit_two_blocks_per_cu_without_scratch(lib):
    # dense_bf16_kernel<T, Ks, TH>: bf16 storage one instantiation per odd kernel size 3 ... 17 and
    # tile height, fp32 storage (three tiles in LDS) per odd kernel size 3 ... 13 at four rows; two
    # blocks per compute unit (256 registers a lane), nothing in the private segment
    meta = {}
    for name, scratch, vgprs, lds in kernel_notes():
        m = re.search(r"dense_bf16_kernelI(f|NS\d_5bf16dE)Li(\d+)ELi(\d+)EE", name)
        if m:
            meta[("f" if m.group(1) == "f" else "b", int(m.group(2)), int(m.group(3)))] = (scratch, vgprs)
    want = {("b", ks, th) for ks in range(3, 18, 2) for th in (4, 8)} | {("f", ks, 4) for ks in range(3, 14, 2)}
    assert set(meta) == want, sorted(set(meta) ^ want)
    for key, (scratch, vgprs) in sorted(meta.items()):
        assert scratch == 0 and vgprs <= 256, (key, scratch, vgprs)


def test_convffn_kernels_use_no_scratch(lib):
    # ffn_stream_kernel runs two blocks per compute unit (256 registers a lane; its 76 KB of LDS
    # are dynamic) with nothing in the private segment; so do the depth-wise branch kernel's four
    # instantiations and the point-wise kernel's eight (storage type x 16-byte fetches x GELU)
    found = {}
    for name, scratch, vgprs, lds in kernel_notes():
        for key in ("ffn_stream_kernel", "ffn_stream_bf16_kernel", "ffn_branch_kernel", "pointwise_kernel", "pointwise_bf16_kernel"):
            if key + "E" in name or key + "I" in name:
                found.setdefault(key, []).append((name, scratch, vgprs))
    assert {k: len(v) for k, v in found.items()} == {"ffn_stream_kernel": 1, "ffn_stream_bf16_kernel": 1, "ffn_branch_kernel": 4,
                                                     "pointwise_kernel": 4, "pointwise_bf16_kernel": 4}, found
    for key, items in found.items():
        for name, scratch, vgprs in items:
            assert scratch == 0 and vgprs <= 256, (name, scratch, vgprs)


def test_three_bf16_terms_hold_an_fp32_value_exactly():
    # The backward's correlation feeds fp32 values to the bf16 matrix instructions as three terms
    # taken by truncation (top 16 bits of the value, of the remainder, of what is left).  The
    # claim the kernel rests on, checked here in numpy: every term is a bf16 value and the three
    # add up to the fp32 value exactly, so that all nine products of two values' terms are exact
    # (values within 2^24 of the smallest normal number lose denormal bits of the third term:
    # an error below 2^-133, checked last).
    rng = np.random.default_rng(77)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * np.float32(10.0) ** rng.integers(-6, 6, 20000),
                        np.array([0.0, -0.0, 1.0, -1.0, 3.0e38, 1.0e-30, np.float32(1) + np.float32(2) ** -23], np.float32)])
    x = x.astype(np.float32)

    def top16(v):
        return (v.view(np.uint32) & np.uint32(0xffff0000)).view(np.float32)

    h = top16(x)
    r1 = x - h
    m = top16(r1)
    r2 = r1 - m
    lo = top16(r2)
    assert np.array_equal(lo, r2)                       # the third term needs no truncation
    s = (h.astype(np.float64) + m.astype(np.float64)) + lo.astype(np.float64)
    assert np.array_equal(s, x.astype(np.float64))
    for t in (h, m, lo):                                # each term is a bf16 value
        assert not (t.view(np.uint32) & np.uint32(0xffff)).any()
    tiny = np.array([1.2e-38, -2.0e-38, 1.0e-36], np.float32)
    th = top16(tiny)
    tm = top16(tiny - th)
    tl = top16(tiny - th - tm)
    err = np.abs(tiny.astype(np.float64) - (th.astype(np.float64) + tm.astype(np.float64) + tl.astype(np.float64)))
    assert err.max() < 2.0 ** -133


def test_two_bf16_terms_hold_a_weight_to_sixteen_mantissa_bits():
    # Conv_fuse, LK^c and the dense large kernel with bf16 storage apply every fp32 weight as
    # hi = bf16(w), lo = bf16(w - hi): the pair must miss w by no more than 2^-17 of |w|.
    from paper_2503_06671_amd import workloads as wk
    rng = np.random.default_rng(78)
    w = (rng.standard_normal(50000) * 10.0 ** rng.integers(-4, 4, 50000)).astype(np.float32)
    hi = wk.bf16_bits_to_f32(wk.f32_to_bf16_bits(w))
    lo = wk.bf16_bits_to_f32(wk.f32_to_bf16_bits(w - hi))
    err = np.abs(w.astype(np.float64) - (hi.astype(np.float64) + lo.astype(np.float64)))
    assert (err <= np.abs(w.astype(np.float64)) * 2.0 ** -17).all()
