"""The polynomial of the FFN epilogue's GeLU (Eq. 1's activation), checked on the CPU against the oracle's erf form.

The kernel evaluates GeLU(v) = ((v + |v|) - x * exp2(q(x))) / 2, x = min(|v|, x_max), in fp32 with fused
multiply-adds; here the same steps run in NumPy (products in float64, rounded to fp32 after every add, which is
what an fma does) on the coefficients parsed from the generated header.
"""
import os
import re

import numpy as np

from oracle import locmoe_oracle as oracle

HEADER = os.path.join(os.path.dirname(__file__), "..", "paper_2401_13920_amd", "csrc", "gelu_coef.h")


def _parse():
    text = open(HEADER).read()
    x_max = float(re.search(r"kGeluXMax = ([-0-9.e+]+)f", text).group(1))
    degree = int(re.search(r"kGeluDegree = (\d+)", text).group(1))
    body = text[text.index("kGeluCoef[kGeluDegree + 1] = {"):]
    coef = [np.float32(m) for m in re.findall(r"^\s+([-0-9.e+]+)f,", body, flags=re.M)]
    assert len(coef) == degree + 1
    return x_max, coef


def _fast_gelu(v, x_max, coef):
    v = v.astype(np.float32)
    x = np.minimum(np.abs(v), np.float32(x_max))
    q = np.full_like(x, coef[-1])
    for c in coef[-2::-1]:
        q = (q.astype(np.float64) * x + np.float64(c)).astype(np.float32)
    h2 = np.exp2(q.astype(np.float64)).astype(np.float32)
    s = (v + np.abs(v)).astype(np.float32)
    return np.float32(0.5) * (s.astype(np.float64) - x.astype(np.float64) * h2).astype(np.float32)


def test_fast_gelu_is_far_inside_the_bf16_rounding_step():
    x_max, coef = _parse()
    rng = np.random.default_rng(5)
    v = np.concatenate([np.linspace(-40.0, 40.0, 400001), rng.normal(0.0, 1.3, 400000), [0.0, -0.0, 1e-30, -1e-30]])
    v = v.astype(np.float32)
    ref = oracle.gelu(v.astype(np.float64))
    got = _fast_gelu(v, x_max, coef).astype(np.float64)
    err = np.abs(got - ref)
    # the element-wise bound of the GPU parity tests is 2^-7 |ref| + 2e-6 after bf16 rounding (2^-9 relative);
    # the approximation itself must stay well below that
    assert np.all(err <= 2.0 ** -13 * np.abs(ref) + 1e-8), (err.max(), v[np.argmax(err)])
    inside = np.abs(v) < x_max
    assert np.max(err[inside] / np.maximum(np.abs(ref[inside]), 1e-300)) < 1e-4
    assert np.all(got[v >= 0] >= 0) and np.all(got[v < 0] <= 0)


def test_fast_gelu_limits():
    x_max, coef = _parse()
    v = np.array([np.inf, -np.inf, np.nan, 100.0, -100.0], dtype=np.float32)
    with np.errstate(invalid="ignore"):
        got = _fast_gelu(v, x_max, coef)
        ref = oracle.gelu(v.astype(np.float64))
    # +inf stays +inf, NaN stays NaN; -inf gives NaN exactly as the defining product (-inf * 0) does
    assert got[0] == np.inf and np.isnan(got[1]) and np.isnan(ref[1]) and np.isnan(got[2])
    assert got[3] == 100.0 and abs(got[4]) < 1e-8
