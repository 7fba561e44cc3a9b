"""CPU oracle for the top-k MoE expert layer, forward and backward.  TEST INFRASTRUCTURE ONLY.

This is the plain definition of the layer written out in numpy fp64 with no blocking, fusion or
reordering.  It exists to check the HIP library and may be imported only by the tests, by the smoke
check and by the CPU-baseline leg of the benchmark; the product path never calls it, and it shares
no code with the HIP path.

What it follows:
  * Section 2.1 of the paper: a gate scores every expert for each token, the token is routed to its
    top-k experts, their outputs are weighted by the scores and summed; dispatch moves token
    embeddings to their experts, combine brings the outputs back.
  * Section 4.2 (asymmetric expert assignment): one GPU may compute only part of the layer's expert
    work; here that share is a half-open range [lo_e, hi_e) over each expert's kept-token list.
  * Section 5 (implementation, gate paragraph): the backward pass from the layer output has two
    branches, one through the experts to their inputs and one through the confidence scores to the
    gate weights and the layer input; both are accumulated into the input gradient.
The paper fixes none of the numerics; the readings used here (softmax over the selected logits,
ties to the lower expert id, ascending-token order inside an expert, capacity drop by list position
with no re-normalisation, exact-erf GELU, SwiGLU = silu(gate) * up) are the ones the benchmark
configurations state.

Pins (tests/test_oracle_*.py): closed forms for the gate and its gradient, brute-force loops for
selection and for the permutation, textbook dense FFN for E=1, identity-expert round trip,
complementary-slice additivity, and central finite differences for every gradient.
Full-size floating-point values have no printed reference in the paper: beyond those pins,
parity unpinned.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erfc

ACT_GELU, ACT_SWIGLU = 0, 1
_SQRT2 = np.sqrt(2.0)
_INV_SQRT_2PI = 1.0 / np.sqrt(2.0 * np.pi)


# ----------------------------------------------------------------------------- activations
def gelu(a):
    """Exact GELU: a * Phi(a), Phi the standard normal CDF (erfc form: accurate in both tails)."""
    return a * (0.5 * erfc(-a / _SQRT2))


def gelu_grad(a):
    """d/da [a Phi(a)] = Phi(a) + a phi(a)."""
    return 0.5 * erfc(-a / _SQRT2) + a * _INV_SQRT_2PI * np.exp(-0.5 * a * a)


def sigmoid(g):
    return 1.0 / (1.0 + np.exp(-g))


def silu(g):
    return g * sigmoid(g)


def silu_grad(g):
    s = sigmoid(g)
    return s * (1.0 + g * (1.0 - s))


# ----------------------------------------------------------------------------- gate (Section 2.1)
def route_logits(x, Wr, bias=None):
    """Confidence scores before normalisation: x @ Wr (+ per-expert bias), fp64."""
    logits = np.asarray(x, dtype=np.float64) @ np.asarray(Wr, dtype=np.float64)
    if bias is not None:
        logits = logits + np.asarray(bias, dtype=np.float64)[None, :]
    return logits


def route_topk(logits, k):
    """Top-k selection and combine weights.

    Selection is made on the logits exactly as given (their dtype is kept for the comparison):
    experts ordered by descending logit, equal logits by ascending id; slot 0 is the best.
    Weights are the softmax over all experts renormalised over the selected ones, which equals
    the softmax over the k selected logits; evaluated in fp64 with the maximum subtracted.
    """
    logits = np.asarray(logits)
    T, E = logits.shape
    assert 1 <= k <= E
    # stable sort of the negated logits: descending value, ties keep ascending expert id
    order = np.argsort(-logits, axis=1, kind="stable")
    idx = order[:, :k].astype(np.int32)
    sel = np.take_along_axis(logits, idx.astype(np.int64), axis=1).astype(np.float64)
    z = np.exp(sel - sel[:, :1])
    w = z / z.sum(axis=1, keepdims=True)
    return idx, w


# ----------------------------------------------------------------------------- dispatch plan
def dispatch_plan(idx, E, capacity=0):
    """Group the T*k assignments by expert.

    Assignment a = t*k + j.  Expert e's list holds its assignments in ascending token order; the
    first min(n_e, capacity) are kept (capacity <= 0: all).  Kept lists are laid out back to back.
    Returns counts[E], kept[E], offsets[E+1], row_of[A] (-1 = dropped), src_of[A] (-1 past the end).
    """
    flat = np.asarray(idx).reshape(-1)
    A = flat.size
    counts = np.zeros(E, dtype=np.int32)
    kept = np.zeros(E, dtype=np.int32)
    offsets = np.zeros(E + 1, dtype=np.int32)
    row_of = np.full(A, -1, dtype=np.int32)
    src_of = np.full(A, -1, dtype=np.int32)
    off = 0
    for e in range(E):
        lst = np.nonzero(flat == e)[0]          # ascending a, hence ascending token
        n_e = lst.size
        m_e = min(n_e, capacity) if capacity > 0 else n_e
        counts[e] = n_e
        kept[e] = m_e
        offsets[e] = off
        row_of[lst[:m_e]] = off + np.arange(m_e)
        src_of[off:off + m_e] = lst[:m_e]
        off += m_e
    offsets[E] = off
    return counts, kept, offsets, row_of, src_of


def clamp_slices(kept, lo=None, hi=None):
    """This GPU's share [lo_e, hi_e) of each kept list; None = everything; clamped to [0, m_e]."""
    kept = np.asarray(kept, dtype=np.int64)
    lo = np.zeros_like(kept) if lo is None else np.clip(np.asarray(lo, dtype=np.int64), 0, kept)
    hi = kept.copy() if hi is None else np.clip(np.asarray(hi, dtype=np.int64), 0, kept)
    hi = np.maximum(hi, lo)
    return lo, hi


def in_share(idx, row_of, offsets, lo, hi):
    """Boolean [A]: assignment is kept and its row lies inside this GPU's share of its expert."""
    flat = np.asarray(idx).reshape(-1).astype(np.int64)
    row_of = np.asarray(row_of, dtype=np.int64)
    pos = row_of - np.asarray(offsets, dtype=np.int64)[flat]
    return (row_of >= 0) & (pos >= lo[flat]) & (pos < hi[flat])


def dispatch_gather(x, src_of, offsets, lo, hi, k):
    """Permuted activations: row r of expert e's share holds token src_of[r] // k.  Other rows NaN."""
    x = np.asarray(x, dtype=np.float64)
    A = len(src_of)
    xp = np.full((A, x.shape[1]), np.nan)
    for e in range(len(lo)):
        r0, r1 = offsets[e] + lo[e], offsets[e] + hi[e]
        xp[r0:r1] = x[np.asarray(src_of[r0:r1]) // k]
    return xp


# ----------------------------------------------------------------------------- expert FFN
def ffn_fwd_block(X, W1, W1b, W2, act):
    """One expert on a block of rows.  GELU: Y = gelu(X W1) W2.  SwiGLU: Y = (silu(X Wg) * X Wu) Wd."""
    if act == ACT_GELU:
        A = X @ W1
        H = gelu(A)
        return {"A": A, "H": H, "Y": H @ W2}
    G = X @ W1
    U = X @ W1b
    H = silu(G) * U
    return {"G": G, "U": U, "H": H, "Y": H @ W2}


def ffn_bwd_block(dY, X, fw, W1, W1b, W2, act):
    """Backward of ffn_fwd_block given its saved intermediates `fw`.

    Returns dX and this block's contribution to the weight gradients.
    """
    dH = dY @ W2.T
    dW2 = fw["H"].T @ dY
    if act == ACT_GELU:
        dA = dH * gelu_grad(fw["A"])
        return {"dH": dH, "dA": dA, "dX": dA @ W1.T, "dW1": X.T @ dA, "dW1b": None, "dW2": dW2}
    dU = dH * silu(fw["G"])
    dG = dH * fw["U"] * silu_grad(fw["G"])
    dX = dG @ W1.T + dU @ W1b.T
    return {"dH": dH, "dG": dG, "dU": dU, "dX": dX, "dW1": X.T @ dG, "dW1b": X.T @ dU, "dW2": dW2}


def expert_ffn_fwd(x_perm, W1, W1b, W2, offsets, lo, hi, act):
    """Every expert on its share of rows.  Rows outside the shares stay NaN."""
    R, f, d = x_perm.shape[0], W1.shape[2], W2.shape[2]
    names = ("A", "H") if act == ACT_GELU else ("G", "U", "H")
    out = {n: np.full((R, f), np.nan) for n in names}
    out["Y"] = np.full((R, d), np.nan)
    for e in range(W1.shape[0]):
        r0, r1 = offsets[e] + lo[e], offsets[e] + hi[e]
        if r1 <= r0:
            continue
        blk = ffn_fwd_block(x_perm[r0:r1], W1[e], None if W1b is None else W1b[e], W2[e], act)
        for n, v in blk.items():
            out[n][r0:r1] = v
    return out


def expert_ffn_bwd(dy_perm, x_perm, fw, W1, W1b, W2, offsets, lo, hi, act):
    """Backward of expert_ffn_fwd; weight gradients sum over the in-share rows only."""
    R, d = x_perm.shape
    dxp = np.full((R, d), np.nan)
    dW1 = np.zeros_like(W1)
    dW1b = None if W1b is None else np.zeros_like(W1b)
    dW2 = np.zeros_like(W2)
    for e in range(W1.shape[0]):
        r0, r1 = offsets[e] + lo[e], offsets[e] + hi[e]
        if r1 <= r0:
            continue
        sub = {n: v[r0:r1] for n, v in fw.items()}
        b = ffn_bwd_block(dy_perm[r0:r1], x_perm[r0:r1], sub, W1[e],
                          None if W1b is None else W1b[e], W2[e], act)
        dxp[r0:r1] = b["dX"]
        dW1[e] = b["dW1"]
        dW2[e] = b["dW2"]
        if dW1b is not None:
            dW1b[e] = b["dW1b"]
    return dxp, dW1, dW1b, dW2


# ----------------------------------------------------------------------------- combine
def combine(y_perm, w, idx, row_of, offsets, lo, hi):
    """out[t] = sum over slots j (in slot order) of w[t,j] * y_perm[row_of[t*k+j]], in-share slots only.

    w=None means unit weights (used for the input-gradient un-permute).
    """
    T, k = np.asarray(idx).shape
    ok = in_share(idx, row_of, offsets, lo, hi).reshape(T, k)
    rows = np.asarray(row_of).reshape(T, k)
    out = np.zeros((T, y_perm.shape[1]))
    for j in range(k):
        t = np.nonzero(ok[:, j])[0]
        wj = 1.0 if w is None else np.asarray(w, dtype=np.float64)[t, j][:, None]
        out[t] += wj * y_perm[rows[t, j]]
    return out


def combine_bwd(d_out, y_perm, w, idx, row_of, offsets, lo, hi):
    """dY[row] = w[a] * dOut[t];  dw[a] = <dOut[t], Y[row]>;  out-of-share slots: dw = 0, row untouched."""
    T, k = np.asarray(idx).shape
    ok = in_share(idx, row_of, offsets, lo, hi).reshape(T, k)
    rows = np.asarray(row_of).reshape(T, k)
    dy = np.full_like(y_perm, np.nan, dtype=np.float64)
    dw = np.zeros((T, k))
    for j in range(k):
        t = np.nonzero(ok[:, j])[0]
        r = rows[t, j]
        dy[r] = np.asarray(w, dtype=np.float64)[t, j][:, None] * d_out[t]
        dw[t, j] = np.einsum("ij,ij->i", d_out[t], y_perm[r])
    return dy, dw


# ----------------------------------------------------------------------------- gate backward
def route_bwd(x, Wr, idx, w, dw):
    """Softmax-over-selected backward, then the linear gate.

    g = sum_j w_j dw_j;  dlogit[t, e_j] = w_j (dw_j - g), zero for unselected experts;
    dWr = x^T dlogits;  the gate's contribution to the input gradient is dlogits Wr^T.
    """
    x = np.asarray(x, dtype=np.float64)
    Wr = np.asarray(Wr, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    T, k = w.shape
    g = (w * dw).sum(axis=1, keepdims=True)
    dsel = w * (dw - g)
    dlogits = np.zeros((T, Wr.shape[1]))
    np.put_along_axis(dlogits, np.asarray(idx, dtype=np.int64), dsel, axis=1)
    return dlogits, x.T @ dlogits, dlogits @ Wr.T


# ----------------------------------------------------------------------------- whole layer
def moe_layer(x, Wr, bias, W1, W1b, W2, d_out, k, act, capacity=0, lo=None, hi=None,
              logits=None, slice_fn=None):
    """Forward and backward of the whole layer on one GPU's share.  All arrays fp64.

    `logits` overrides the gate's own logits for the top-k decision and the weights (used to
    replay routing from logits computed elsewhere).  `slice_fn(kept) -> (lo, hi)` may supply the
    share once the kept counts are known.
    Loss convention for the backward: L = sum(out * d_out).
    """
    f64 = lambda a: None if a is None else np.asarray(a, dtype=np.float64)
    x, Wr, W1, W1b, W2, d_out = map(f64, (x, Wr, W1, W1b, W2, d_out))
    E = Wr.shape[1]
    r = {}
    r["logits"] = route_logits(x, Wr, bias)
    used = r["logits"] if logits is None else logits
    r["idx"], r["w"] = route_topk(used, k)
    r["counts"], r["kept"], r["offsets"], r["row_of"], r["src_of"] = dispatch_plan(r["idx"], E, capacity)
    if slice_fn is not None:
        lo, hi = slice_fn(r["kept"])
    lo, hi = clamp_slices(r["kept"], lo, hi)
    r["lo"], r["hi"] = lo, hi
    r["x_perm"] = dispatch_gather(x, r["src_of"], r["offsets"], lo, hi, k)
    fw = expert_ffn_fwd(r["x_perm"], W1, W1b, W2, r["offsets"], lo, hi, act)
    r["fw"] = fw
    r["out"] = combine(fw["Y"], r["w"], r["idx"], r["row_of"], r["offsets"], lo, hi)
    # backward
    r["dy_perm"], r["dw"] = combine_bwd(d_out, fw["Y"], r["w"], r["idx"], r["row_of"], r["offsets"], lo, hi)
    saved = {n: v for n, v in fw.items() if n != "Y"}
    r["dx_perm"], r["dW1"], r["dW1b"], r["dW2"] = expert_ffn_bwd(
        r["dy_perm"], r["x_perm"], saved, W1, W1b, W2, r["offsets"], lo, hi, act)
    r["dx_experts"] = combine(r["dx_perm"], None, r["idx"], r["row_of"], r["offsets"], lo, hi)
    r["dlogits"], r["dWr"], r["dx_gate"] = route_bwd(x, Wr, r["idx"], r["w"], r["dw"])
    r["dx"] = r["dx_experts"] + r["dx_gate"]
    return r
