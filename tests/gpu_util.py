"""Helpers for the GPU parity tests: upload a workload, run the HIP path, run the oracle, compare."""
from __future__ import annotations

import numpy as np

from oracle import moe_oracle as O
from paper_2504_03871_amd import synth as S

# fp16 keeps 11 significand bits against the 8 of bf16: the same chain of storage roundings (saved activations,
# y, dy, dA, dx) is 8 times finer, hence the bf16 tolerance divided by 8
TOL = {S.DT_F32: 1e-5, S.DT_BF16: 2e-2, S.DT_F16: 2.5e-3}
SENTINEL = 12288.0   # 1.5 * 2^13, exact in bf16 and fp32


def to_dev(arr_f32, bits, device, dtype):
    import torch
    if dtype == S.DT_BF16:
        return torch.from_numpy(bits.view(np.int16).copy()).to(device).view(torch.bfloat16)
    if dtype == S.DT_F16:
        return torch.from_numpy(bits.view(np.int16).copy()).to(device).view(torch.float16)
    return torch.from_numpy(np.ascontiguousarray(arr_f32, dtype=np.float32)).to(device)


def make_layer(w: S.Workload, inp: dict, device="cuda:0"):
    from paper_2504_03871_amd.layer import MoELayer
    import torch
    L = MoELayer(w.T, w.d, w.f, w.E, w.k, dtype=w.dtype, act=w.act, capacity=w.capacity, device=device)
    for name, attr in (("x", "x"), ("W1", "W1"), ("W2", "W2"), ("d_out", "d_out"), ("W1b", "W1b")):
        if name in inp:
            getattr(L, attr).copy_(to_dev(inp[name], inp.get(name + "_bits"), device, w.dtype))
    L.Wr.copy_(torch.from_numpy(inp["Wr"]).to(device))
    if inp.get("bias") is not None:
        L.bias = torch.from_numpy(inp["bias"]).to(device)
    return L


def fill_sentinels(L):
    """Every output buffer starts at a sentinel so that untouched rows can be recognised."""
    for name in ("x_perm", "y_perm", "out", "dy_perm", "dx_perm", "dx", "dW1", "dW2", "dW1b", "d_logits", "dWr",
                 "d_topk_w", "logits", "topk_w"):
        t = getattr(L, name)
        if t is not None:
            t.fill_(SENTINEL)
    for i in range(3 if L.act == 1 else 2):
        L.saved_plane(i).fill_(SENTINEL)
    for name in ("topk_idx", "counts", "kept", "offsets", "row_of", "src_of"):
        getattr(L, name).fill_(-7)


def host(t):
    import torch
    if t.dtype in (torch.bfloat16, torch.float16):
        return t.float().cpu().numpy().astype(np.float64)
    a = t.cpu().numpy()
    return a.astype(np.float64) if a.dtype == np.float32 else a


def rel_err(got, ref, scale=None):
    """(relative L2 error, max abs error / max abs ref) over the finite entries of ref.

    `scale` (same shape as ref, or None) is a second yardstick for outputs that are sums with cancellation:
    the size each entry would have without it.  The denominators are then the larger of the reference's own
    norm and the scale's, so that a reference whose few entries all happen to cancel is not the measure.
    """
    m = np.isfinite(ref)
    g, r = got[m], ref[m]
    den = np.linalg.norm(r)
    mx = np.abs(r).max() if r.size else 0.0
    if scale is not None:
        den = max(den, np.linalg.norm(scale[m]))
        mx = max(mx, np.abs(scale[m]).max() if r.size else 0.0)
    l2 = np.linalg.norm(g - r) / den if den > 0 else np.linalg.norm(g - r)
    ma = np.abs(g - r).max() / mx if mx > 0 else (np.abs(g - r).max() if r.size else 0.0)
    return l2, ma


def assert_close(name, got, ref, tol, scale=None):
    assert got.shape == ref.shape, f"{name}: shape {got.shape} vs {ref.shape}"
    assert np.isfinite(got[np.isfinite(ref)]).all(), f"{name}: non-finite values"
    l2, ma = rel_err(got, ref, scale)
    assert l2 <= tol and ma <= tol, f"{name}: rel L2 {l2:.3e}, max-abs/max {ma:.3e} > {tol:g}"
    return l2, ma


def dot_scale(d_out, y_perm, idx, row_of, offsets, lo, hi):
    """[T, k]: sqrt(sum_i (d_out[t, i] * y_perm[row, i])^2) of every in-share slot, 0 elsewhere: the size that the
    rounding errors of the d products of d_topk_w[t, j] = <d_out[t], y_perm[row]> add up to when they are
    independent (each product is good to the storage type's unit roundoff), whatever the sum cancels to."""
    T, k = np.asarray(idx).shape
    ok = O.in_share(idx, row_of, offsets, lo, hi).reshape(T, k)
    rows = np.asarray(row_of).reshape(T, k)
    sc = np.zeros((T, k))
    for j in range(k):
        t = np.nonzero(ok[:, j])[0]
        sc[t, j] = np.sqrt(((np.asarray(d_out, dtype=np.float64)[t] * y_perm[rows[t, j]]) ** 2).sum(axis=1))
    return sc


def run_oracle(w: S.Workload, inp: dict, gpu_logits=None, lo=None, hi=None, slice_fn=None):
    return O.moe_layer(inp["x"], inp["Wr"], inp.get("bias"), inp["W1"], inp.get("W1b"), inp["W2"], inp["d_out"],
                       w.k, w.act, capacity=w.capacity, lo=lo, hi=hi, logits=gpu_logits, slice_fn=slice_fn)


def untouched_rows(t, live_mask):
    """True if every row not in live_mask still holds the sentinel."""
    a = host(t)
    dead = ~live_mask
    return bool((a[dead] == SENTINEL).all())
