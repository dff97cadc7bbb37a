"""CPU pin of a claim the ConvFFN kernels' comments make: the rational approximation of erf
they use (Abramowitz and Stegun, Handbook of Mathematical Functions, 7.1.26), evaluated in
float32 in the kernels' order of operations, keeps GELU within 6e-7 of its erf definition
(and within 3e-7 |v|) - far inside the 1e-5 parity bar.  The GPU test of the same name in
tests/test_gpu_ffn.py measures the kernels themselves."""
import math

import numpy as np


def test_rational_erf_keeps_gelu_within_its_stated_error():
    f = np.float32
    v = np.linspace(-12.0, 12.0, 600001).astype(f)
    a = np.abs(v) * f(0.70710678118654752440)
    t = (f(1) / (f(0.3275911) * a + f(1))).astype(f)
    q = f(1.061405429) * t + f(-1.453152027)
    for c in (1.421413741, -0.284496736, 0.254829592):
        q = (q * t + f(c)).astype(f)
    e = np.exp2((a * a * f(-1.44269504088896340736)).astype(f)).astype(f)
    erf_a = (f(1) - (q * t).astype(f) * e).astype(f)
    h = f(0.5) * v
    g = (np.abs(h) * erf_a + h).astype(np.float64)
    ref = np.array([0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0))) for x in v.astype(np.float64)])
    err = np.abs(g - ref)
    assert err.max() <= 6e-7, err.max()
    assert (err <= 3e-7 * np.maximum(np.abs(v), 1e-2)).all()
    assert g[np.abs(v) == 0].tolist() == [0.0] * int((v == 0).sum())
