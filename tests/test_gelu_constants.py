"""The GELU polynomial of the kernels (csrc/nf_common.h): its constants are the committed fit's, and in float32
arithmetic it stays within 1e-6 of the exact 0.5 x (1 + erf(x / sqrt 2))."""
import importlib.util
import math
import os
import re

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2009_13062_amd", "csrc")


def header_coefficients():
    """a^0 .. a^6, read from the Horner chain of gelu_erf."""
    text = open(os.path.join(CSRC, "nf_common.h")).read()
    body = text[text.index("float gelu_erf(float v)"):]
    body = body[:body.index("return v *")]
    first = re.search(r"fmaf\(([-0-9.e+]+)f, a, ([-0-9.e+]+)f\)", body)
    rest = re.findall(r"g = fmaf\(g, a, ([-0-9.e+]+)f\)", body)
    high_to_low = [float(first.group(1)), float(first.group(2))] + [float(x) for x in rest]
    assert len(high_to_low) == 7
    return high_to_low[::-1]


def fit_module():
    spec = importlib.util.spec_from_file_location("gelu_fit", os.path.join(CSRC, "gelu_fit.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    return m


def test_header_constants_are_the_committed_fit():
    m = fit_module()
    assert header_coefficients() == m.fit()


def test_polynomial_error_bound_against_math_erf():
    m = fit_module()
    c = header_coefficients()
    v = np.concatenate([np.linspace(-12, 12, 400001), np.linspace(-1e-3, 1e-3, 2001), [-30.0, 30.0, 0.0]])
    exact = np.array([0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0))) for x in v])
    got = m.gelu_poly_f32(v, c).astype(np.float64)
    err = np.abs(got - exact)
    assert err.max() < 1e-6, (err.max(), v[err.argmax()])
    # far tails (|v| is clamped to 8 inside the polynomial): v itself, and v times a tail below 1e-15
    assert abs(got[-3]) < 1e-12 and got[-2] == 30.0
