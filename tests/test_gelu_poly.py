"""The constants of the per-token aggregator's GELU (host logic, no GPU): the fit script beside the
kernel reproduces them, and a float32 evaluation in the kernel's order stays within 1e-7 of erfc/2,
i.e. the polynomial is the exact-erf GELU to fp32 accuracy."""
import importlib.util
import os
import re

import numpy as np
from scipy import special

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2509_21354_amd", "csrc")


def _fit_module():
    spec = importlib.util.spec_from_file_location("fit_gelu_poly", os.path.join(CSRC, "fit_gelu_poly.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def _kernel_constants():
    src = open(os.path.join(CSRC, "pool_token_mfma.hip")).read()
    body = src[src.index("float add_gelu_poly(float acc, float z)"):]
    body = body[:body.index("__builtin_amdgcn_exp2f")]
    u_max = float(re.search(r"fmed3f\(fabsf\(z\), 0\.f, ([0-9.]+)f\)", body).group(1))
    first = re.search(r"float q = (-?[0-9.e+-]+)f;", body).group(1)
    rest = re.findall(r"q = fmaf\(q, u, (-?[0-9.e+-]+)f\);", body)
    assert rest[-1] == "-1.0"                       # the last step adds log2(1/2)
    return np.array([float(x) for x in reversed([first] + rest[:-1])], dtype=np.float32), u_max      # c0 .. c6


def test_kernel_constants_are_the_fit_and_accurate():
    m = _fit_module()
    c_kernel, u_max = _kernel_constants()
    c_fit = m.coefficients().astype(np.float32)
    assert len(c_kernel) == m.DEGREE and abs(u_max - m.U_MAX) < 1e-6
    assert np.allclose(c_kernel, c_fit, rtol=2e-6, atol=0)
    u = np.linspace(0.0, 12.0, 200001)
    assert np.abs(m.tail_f32(u, c_kernel) - special.erfc(u / np.sqrt(2.0)) * 0.5).max() < 1e-7
    # slope at 0: d/du log2 erfc(u / sqrt 2) = -sqrt(2 / pi) log2 e
    assert abs(c_kernel[0] + np.sqrt(2.0 / np.pi) * np.log2(np.e)) < 1e-5
    # GELU through it, in the kernel's form max(z, 0) - |z| E(|z|), against the erf form in double precision
    z = np.linspace(-12.0, 12.0, 100001)
    E = m.tail_f32(np.abs(z), c_kernel).astype(np.float64)
    gelu = np.maximum(z, 0.0) - np.abs(z) * E
    want = 0.5 * z * (1.0 + special.erf(z / np.sqrt(2.0)))
    assert np.abs(gelu - want).max() < 2e-7
