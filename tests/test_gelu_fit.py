"""The fitted GELU of the bf16 GEMM epilogue against the oracle's exact GELU (CPU, fp32 emulation).

The coefficients are read from the kernel source, so a typo there fails here without a GPU."""
import os
import re

import numpy as np

from oracle import moe_oracle as O

SRC = os.path.join(os.path.dirname(__file__), "..", "paper_2504_03871_amd", "csrc", "gemm_bf16_kernel.h")


def _coefficients():
    text = open(SRC).read()
    body = text[text.index("float gelu_fast(float a)"):]
    body = body[:body.index("return")]
    lead = re.search(r"float p = (-?[0-9.e+-]+)f;", body).group(1)
    rest = re.findall(r"p = fmaf\(p, x, (-?[0-9.e+-]+)f\);", body)
    assert len(rest) == 6
    return [np.float32(lead)] + [np.float32(c) for c in rest]


def gelu_fit_f32(a):
    c = _coefficients()
    a = a.astype(np.float32)
    x = np.minimum(np.abs(a), np.float32(6.0))
    p = np.full_like(x, c[0])
    for ck in c[1:]:
        p = (p * x + ck).astype(np.float32)
    t = np.exp2((x * p - np.float32(1.0)).astype(np.float32)).astype(np.float32)
    return (np.maximum(a, np.float32(0)) - np.abs((a * t).astype(np.float32))).astype(np.float32)


def test_fitted_gelu_matches_exact_gelu():
    a = np.linspace(-40.0, 40.0, 800001)
    ref = O.gelu(a)
    got = gelu_fit_f32(a).astype(np.float64)
    assert np.max(np.abs(got - ref)) < 1.2e-5          # |a| up to 40; below 2e-6 inside [-12, 12]
    m = np.abs(a) <= 12
    assert np.max(np.abs(got[m] - ref[m])) < 2e-6
    m = (np.abs(a) <= 6) & (a != 0)
    assert np.max(np.abs(got[m] - ref[m]) / np.abs(ref[m])) < 3e-5
