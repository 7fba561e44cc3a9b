"""The fp16 gate kernels feed bf16 matrix instructions with fp16 activations split into two bf16 terms
(csrc/route.hip, XTerms<f16>): the first 8 significant bits (the fp32 image truncated to its upper 16 bits) and the
rest.  This checks the claim the kernels rest on, for every fp16 bit pattern: both terms are bf16 numbers (their
fp32 images have zero lower halves) and their sum is the fp16 value exactly."""
import numpy as np


def test_every_fp16_value_is_the_sum_of_two_bf16_numbers():
    bits = np.arange(1 << 16, dtype=np.uint16)
    f = bits.view(np.float16).astype(np.float32)
    finite = np.isfinite(f)
    u = f.view(np.uint32)
    hi = (u & np.uint32(0xFFFF0000)).view(np.float32)           # truncation to bf16
    with np.errstate(invalid="ignore"):
        lo = f - hi                                               # fp32 subtraction
    assert ((lo.view(np.uint32)[finite] & 0xFFFF) == 0).all()     # the rest is a bf16 number as it stands
    s = hi.astype(np.float64) + lo.astype(np.float64)
    assert (s[finite] == f.astype(np.float64)[finite]).all()
    # and the rest is small: at most 3 significant bits below the first 8
    nz = finite & (f != 0)
    assert (np.abs(lo[nz]) <= np.abs(f[nz]) * 2.0 ** -7).all()
    # an infinity is its own first term (the kernels then take 0 for the rest instead of inf - inf)
    inf = np.isinf(f)
    assert (hi[inf] == f[inf]).all()
