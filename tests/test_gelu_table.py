"""The GELU tables of the bf16 GEMM epilogues: index mapping and clamping, emulated on the CPU.

The constants are read from the kernel header, the table entries come from the oracle's exact functions, and
every bf16 bit pattern is pushed through the same index arithmetic the epilogue uses."""
import os
import re

import numpy as np

from oracle import moe_oracle as O

HDR = os.path.join(os.path.dirname(__file__), "..", "paper_2504_03871_amd", "csrc", "gemm.h")


def _constants():
    text = open(HDR).read()
    exp0 = int(re.search(r"GELU_TAB_EXP0 = (\d+);", text).group(1))
    hi, lo = re.search(r"GELU_TAB_NMAG = \((\d+) - (\d+)\) \* 128;", text).groups()
    floats = int(re.search(r"GELU_TAB_FLOATS = (\d+);", text).group(1))
    return exp0, (int(hi) - int(lo)) * 128, floats


def _bf16_value(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _lookup(table, bits, exp0, nmag):
    m = np.clip((bits & 0x7FFF).astype(np.int64) - (exp0 << 7), 0, nmag - 1)
    return table[m + (bits >> 15).astype(np.int64) * nmag]


def test_tables_cover_every_bf16_number():
    exp0, nmag, floats = _constants()
    assert 2 * nmag <= floats and (floats * 4) % (512 * 16) == 0      # whole block-wide 16-byte loads
    idx = np.arange(2 * nmag)
    arg = _bf16_value(((idx % nmag) + (exp0 << 7)) | np.where(idx >= nmag, 0x8000, 0))
    assert arg[0] == 2.0 ** -16 and arg[nmag - 1] < 8.0 and arg[nmag] == -(2.0 ** -16)
    phi_tab = O.gelu(arg) / arg
    phi_tab[nmag - 1], phi_tab[2 * nmag - 1] = 1.0, 0.0               # the last magnitude stands for all larger ones
    grad_tab = O.gelu_grad(arg)
    bits = np.arange(65536, dtype=np.uint32)
    v = _bf16_value(bits)
    ok = np.isfinite(v)
    bits, v = bits[ok], v[ok]
    # backward: the derivative at the stored number
    assert np.max(np.abs(_lookup(grad_tab, bits, exp0, nmag) - O.gelu_grad(v))) < 1.3e-5
    # forward: h = a * Phi(v) with a = v here; zero stays zero, large arguments pass through
    h = v * _lookup(phi_tab, bits, exp0, nmag)
    ref = O.gelu(v)
    assert np.all(np.abs(h - ref) <= 1.3e-5 * np.abs(ref) + 1e-14)
    assert np.all(h[v >= 8.0] == v[v >= 8.0]) and np.all(h[v <= -7.96875] == 0.0)
    assert h[bits == 0][0] == 0.0 and h[bits == 0x8000][0] == 0.0
