"""The constants of the chunk-MLP kernel's erf-form GELU (csrc/fc_mlp.hip:
Phi(-|v|) = exp2(P(|v|)), P of degree 6) against the definition, on the CPU:
the polynomial is read from the kernel source, evaluated the way the kernel
evaluates it (fp32 Horner steps, fp32 exp2, clamp) and compared with
v * Phi(v) from math.erfc.  The bound is what the derived parity tolerance of
tests/parity_util.py allows the activation (H_ABS), with a wide margin."""

import math
import os
import re

import numpy as np

from conftest import ROOT


def _constants():
    src = open(os.path.join(ROOT, "paper_2503_08461_amd", "csrc", "fc_mlp.hip")).read()
    vals = {}
    for name, text in re.findall(r"#define FC_GELU_TAIL_(\w+) (-?[0-9.e+-]+)f", src):
        vals[name] = float(text)
    assert sorted(vals) == ["CLAMP", "P0", "P1", "P2", "P3", "P4", "P5", "P6"]
    return [vals["P%d" % k] for k in range(7)], vals["CLAMP"]


def _kernel_gelu(v32, coeff, clamp):
    c = [np.float32(t) for t in coeff]
    a = np.minimum(np.abs(v32), np.float32(clamp))
    p = np.full_like(a, c[6])
    for k in range(5, -1, -1):
        p = (p * a + c[k]).astype(np.float32)     # (an fma rounds once: at least as accurate)
    vq = (v32 * np.exp2(p).astype(np.float32)).astype(np.float32)
    return np.where(v32 < 0, vq, (v32 - vq).astype(np.float32))


def test_tail_polynomial_reproduces_gelu_by_its_definition():
    coeff, clamp = _constants()
    v = np.concatenate([np.linspace(-60, 60, 240001),
                        np.linspace(-1, 1, 20001),
                        np.array([0.0, -0.0, 8.5, -8.5, 8.4999, 1e-8, -1e-8, 65504.0, -65504.0])])
    v32 = v.astype(np.float32)
    exact = np.array([x * 0.5 * math.erfc(-x / math.sqrt(2.0)) for x in v32.astype(np.float64)])
    got = _kernel_gelu(v32, coeff, clamp).astype(np.float64)
    err = np.abs(got - exact)
    # absolute: two orders of magnitude inside the activation allowance of the parity bound
    assert err.max() < 1e-6, (err.max(), v32[np.argmax(err)])
    # and relative to the magnitude of the input: no term is lost for large |v|
    assert (err / np.maximum(np.abs(v32.astype(np.float64)), 1.0)).max() < 5e-7
    assert got[np.where(v32 == 65504.0)[0][0]] == 65504.0
    assert abs(got[np.where(v32 == -65504.0)[0][0]]) < 1e-10


def test_tail_at_fixed_points():
    """Phi(-x) itself at a few points of a normal table, through exp2(P(x))."""
    coeff, clamp = _constants()
    for x, phi in ((0.0, 0.5), (1.0, 0.158655254), (1.96, 0.024997895), (3.0, 0.001349898)):
        p = sum(c * x ** k for k, c in enumerate(coeff))
        assert abs(2.0 ** p - phi) < 2e-7 * max(1.0, phi / 0.0013), (x, 2.0 ** p, phi)
