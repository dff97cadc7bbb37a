"""MI355X-native ConvAttn forward pass (ESC paper, Sec. 3, Eq. 4).

The compute lives in hand-written HIP kernels behind a C ABI
(include/esc_convattn.h, built into csrc/libesc_convattn.so); `binding` is the
thin ctypes layer over it and `workloads` the seeded synthetic inputs.  Nothing
is loaded at import time; the first call into `binding` loads the library and
raises if it has not been built.
"""
__all__ = ["binding", "workloads"]
