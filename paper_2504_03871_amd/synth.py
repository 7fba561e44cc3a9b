"""Seeded synthetic inputs for the MoE expert layer (shared by tests, bench and the CPU checker).

This module holds no arithmetic of the method itself: it only draws numbers, rounds them to the
storage type and describes the workloads.  Every tensor is a pure function of (seed, element index),
so any slice of any tensor can be regenerated independently and the GPU path and the CPU checker
consume byte-identical inputs.

Generator: a SplitMix64 counter stream (the 64-bit finaliser published by Steele, Lea and Flood,
"Fast splittable pseudorandom number generators", 2014) feeds a Box-Muller transform evaluated in
fp64; element i of a tensor uses counters 2i and 2i+1 and keeps the cosine branch only.

Workload shapes follow the five benchmark configurations of this build (hidden sizes 1024/2048 echo
Table 2 of the paper, the Mixtral-like shape echoes the module settings of Fig. 2, top-2 routing is
the setting of Section 6.1).
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np

BASE_SEED = 250403871

# tensor ids (seed = BASE_SEED + 1000 * config_id + tensor_id)
TID_X, TID_WR, TID_W1, TID_W1B, TID_W2, TID_DOUT = 0, 1, 2, 3, 4, 5

ACT_GELU, ACT_SWIGLU = 0, 1
DT_F32, DT_BF16, DT_F16 = 0, 1, 2

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, counters: np.ndarray) -> np.ndarray:
    """SplitMix64 output number `counters` (uint64 array, 0-based) of the stream started at `seed`."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed % (1 << 64)) + (counters.astype(np.uint64) + np.uint64(1)) * _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def _unit_open(z: np.ndarray) -> np.ndarray:
    """Top 53 bits of z mapped to the open interval (0, 1)."""
    return ((z >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal_block(seed: int, start: int, count: int, std: float = 1.0) -> np.ndarray:
    """Elements [start, start+count) of the N(0, std^2) tensor with this seed, as fp64."""
    i = np.arange(start, start + count, dtype=np.uint64)
    u1 = _unit_open(splitmix64(seed, i * np.uint64(2)))
    u2 = _unit_open(splitmix64(seed, i * np.uint64(2) + np.uint64(1)))
    return np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * math.pi) * u2) * std


def normal_f32(seed: int, shape, std: float = 1.0, threads: int = 8, chunk: int = 1 << 22) -> np.ndarray:
    """Whole tensor as fp32 (the fp64 draw rounded once to fp32), generated in parallel chunks."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)

    def fill(s):
        e = min(n, s + chunk)
        out[s:e] = normal_block(seed, s, e - s, std)

    starts = list(range(0, n, chunk))
    if len(starts) <= 1 or threads <= 1:
        for s in starts:
            fill(s)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, starts))
    return out.reshape(shape)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round to nearest, ties to even); returns the 16-bit patterns."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_f16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to IEEE half precision (round to nearest, ties to even); returns the 16-bit patterns."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def f16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return bits.view(np.float16).astype(np.float32)


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration.  `cid` selects the seeds; the rest is the layer shape."""
    name: str
    cid: int
    T: int
    d: int
    f: int
    E: int
    k: int
    act: int = ACT_GELU
    dtype: int = DT_BF16
    capacity_factor: float = 0.0      # 0 = unlimited
    zipf_s: float = 0.0               # router bias -s*ln(e+1); 0 = none
    partial: bool = False             # config-4 style slices (upper half of the experts: last 40 %)

    @property
    def capacity(self) -> int:
        """Rows kept per expert: ceil(cf * T * k / E) in exact rational arithmetic; 0 = unlimited."""
        if self.capacity_factor <= 0:
            return 0
        num, den = float(self.capacity_factor).as_integer_ratio()
        a = num * self.T * self.k
        b = den * self.E
        return -((-a) // b)

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "cfg0": Workload("cfg0", 0, T=512, d=128, f=256, E=8, k=2, dtype=DT_F32),
    "cfg1": Workload("cfg1", 1, T=8192, d=1024, f=4096, E=8, k=2),
    "cfg2": Workload("cfg2", 2, T=16384, d=2048, f=8192, E=16, k=2, zipf_s=1.2),
    "cfg3": Workload("cfg3", 3, T=32768, d=4096, f=14336, E=8, k=2, act=ACT_SWIGLU),
    "cfg4": Workload("cfg4", 4, T=16384, d=2048, f=8192, E=32, k=4, capacity_factor=1.25, partial=True),
    # cfg4 with the skewed router of cfg2, so that capacity overflow really drops tokens
    "cfg4z": Workload("cfg4z", 4, T=16384, d=2048, f=8192, E=32, k=4, capacity_factor=1.25,
                      partial=True, zipf_s=1.2),
    # many small experts (the model trend Section 6.2 of the paper says favours it): 128 and 256 experts,
    # top-8, narrow FFNs; a few hundred rows per expert, so partly filled row tiles dominate
    "cfg5": Workload("cfg5", 5, T=8192, d=2048, f=1024, E=128, k=8, act=ACT_SWIGLU),
    "cfg6": Workload("cfg6", 6, T=8192, d=2048, f=1024, E=256, k=8),
}


def _seed(w: Workload, tid: int) -> int:
    return BASE_SEED + 1000 * w.cid + tid


def router_bias(w: Workload):
    """Additive per-expert logit bias: log of the Zipf(s) rank weight, normaliser dropped."""
    if w.zipf_s <= 0:
        return None
    return (-w.zipf_s * np.log(np.arange(1, w.E + 1, dtype=np.float64))).astype(np.float32)


def make_inputs(w: Workload, threads: int = 8) -> dict:
    """All input tensors of one workload.

    Returns fp32 arrays holding the values both sides consume: for bf16 and fp16 workloads x, the
    expert weights and the upstream gradient are already rounded to the storage type (and
    `<name>_bits` holds the 16-bit patterns to upload); the router weight and bias stay fp32.
    """
    out = {}
    x = normal_f32(_seed(w, TID_X), (w.T, w.d), 1.0, threads)
    wr = normal_f32(_seed(w, TID_WR), (w.d, w.E), 1.0 / math.sqrt(w.d), threads)
    w1 = normal_f32(_seed(w, TID_W1), (w.E, w.d, w.f), 0.02, threads)
    w2 = normal_f32(_seed(w, TID_W2), (w.E, w.f, w.d), 0.02, threads)
    dout = normal_f32(_seed(w, TID_DOUT), (w.T, w.d), 1.0, threads)
    tensors = {"x": x, "W1": w1, "W2": w2, "d_out": dout}
    if w.act == ACT_SWIGLU:
        tensors["W1b"] = normal_f32(_seed(w, TID_W1B), (w.E, w.d, w.f), 0.02, threads)
    for name, a in tensors.items():
        if w.dtype == DT_BF16:
            bits = f32_to_bf16_bits(a)
            out[name + "_bits"] = bits
            out[name] = bf16_bits_to_f32(bits)
        elif w.dtype == DT_F16:
            bits = f32_to_f16_bits(a)
            out[name + "_bits"] = bits
            out[name] = f16_bits_to_f32(bits)
        else:
            out[name] = a
    out["Wr"] = wr
    out["bias"] = router_bias(w)
    return out


def partial_slices(w: Workload, kept: np.ndarray):
    """Per-expert [lo, hi) over the kept list for this GPU's share.

    Full workloads: every expert in full.  Partial workloads: the lower half of the experts in
    full, the upper half only on the last floor(2*m_e/5) rows of each one's kept list.
    """
    kept = np.asarray(kept, dtype=np.int64)
    lo = np.zeros(w.E, dtype=np.int32)
    hi = kept.astype(np.int32).copy()
    if w.partial:
        for e in range(w.E // 2, w.E):
            cnt = (2 * int(kept[e])) // 5
            lo[e] = int(kept[e]) - cnt
    return lo, hi
