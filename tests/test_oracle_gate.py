"""Pins for the oracle's gate: closed forms, invariants, brute force (Section 2.1 of the paper)."""
import math

import numpy as np
import pytest

from oracle import moe_oracle as O


def test_closed_form_ln_logits():
    # logits ln1..ln4, k=2: softmax over the two best = 4/(4+3), 3/(4+3)
    logits = np.log(np.array([[1.0, 2.0, 3.0, 4.0]]))
    idx, w = O.route_topk(logits, 2)
    assert idx.tolist() == [[3, 2]]
    np.testing.assert_allclose(w, [[4 / 7, 3 / 7]], rtol=1e-15)


def test_all_equal_logits_pick_lowest_ids():
    for dt in (np.float32, np.float64):
        idx, w = O.route_topk(np.full((3, 6), 0.25, dtype=dt), 3)
        assert idx.tolist() == [[0, 1, 2]] * 3
        np.testing.assert_allclose(w, 1 / 3, rtol=1e-15)


def test_tie_at_top_and_signed_zero():
    idx, _ = O.route_topk(np.array([[0.5, 2.0, 2.0, -1.0]]), 2)
    assert idx.tolist() == [[1, 2]]
    idx, _ = O.route_topk(np.array([[1.0, 3.0, 0.0, 3.0]]), 3)
    assert idx.tolist() == [[1, 3, 0]]
    # -0.0 and +0.0 compare equal: the lower id wins whichever sign it carries
    idx, _ = O.route_topk(np.array([[0.0, -0.0, -5.0]], dtype=np.float32), 1)
    assert idx.tolist() == [[0]]
    idx, _ = O.route_topk(np.array([[-0.0, 0.0, -5.0]], dtype=np.float32), 1)
    assert idx.tolist() == [[0]]


def test_k_equals_E_is_full_softmax():
    rng = np.random.default_rng(1)
    l = rng.normal(size=(50, 7))
    idx, w = O.route_topk(l, 7)
    full = np.exp(l) / np.exp(l).sum(1, keepdims=True)       # textbook softmax, no max-shift
    np.testing.assert_allclose(w, np.take_along_axis(full, idx.astype(np.int64), 1), rtol=1e-13)


def test_invariants_random():
    rng = np.random.default_rng(2)
    l = rng.normal(size=(2000, 16)).astype(np.float32)
    k = 4
    idx, w = O.route_topk(l, k)
    assert idx.dtype == np.int32 and idx.min() >= 0 and idx.max() < 16
    assert all(len(set(r)) == k for r in idx.tolist())
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-14)
    assert (np.diff(w, axis=1) <= 0).all()                   # slot order = descending weight
    # shift invariance of the weights and of the selection.  Shift by a power of two well above
    # the logits so that the fp64 addition is exact.
    idx2, w2 = O.route_topk(l.astype(np.float64) + 1024.0, k)
    assert (idx2 == idx).all()
    np.testing.assert_allclose(w2, w, rtol=1e-12)
    # renormalised full softmax equals softmax over the selected logits
    p = np.exp(l.astype(np.float64))
    p /= p.sum(1, keepdims=True)
    ps = np.take_along_axis(p, idx.astype(np.int64), 1)
    np.testing.assert_allclose(ps / ps.sum(1, keepdims=True), w, rtol=1e-12)


def _brute_topk(row, k):
    """Selection by repeated scan: best remaining value, first occurrence wins."""
    taken, out = set(), []
    for _ in range(k):
        best = None
        for e, v in enumerate(row):
            if e in taken:
                continue
            if best is None or v > row[best]:
                best = e
        taken.add(best)
        out.append(best)
    return out


def test_brute_force_with_forced_ties():
    rng = np.random.default_rng(3)
    vals = np.array([-1.0, 0.0, 0.5, 2.0], dtype=np.float32)
    for _ in range(4000):
        E = int(rng.integers(1, 9))
        k = int(rng.integers(1, E + 1))
        row = vals[rng.integers(0, 4, size=E)]
        idx, _ = O.route_topk(row[None, :], k)
        assert idx[0].tolist() == _brute_topk(row.tolist(), k)
    for _ in range(2000):
        E = int(rng.integers(2, 12))
        k = int(rng.integers(1, E + 1))
        row = rng.normal(size=E).astype(np.float32)
        idx, _ = O.route_topk(row[None, :], k)
        assert idx[0].tolist() == _brute_topk(row.tolist(), k)


def test_route_logits_matches_loops():
    rng = np.random.default_rng(4)
    x = rng.normal(size=(5, 7))
    Wr = rng.normal(size=(7, 3))
    b = rng.normal(size=3)
    got = O.route_logits(x, Wr, b)
    for t in range(5):
        for e in range(3):
            s = b[e]
            for i in range(7):
                s += x[t, i] * Wr[i, e]
            assert got[t, e] == pytest.approx(s, rel=1e-13, abs=1e-14)


def test_gate_backward_closed_form():
    # w = (4/7, 3/7), dw = (1, 0): g = 4/7, dlogit = (4/7*(1-4/7), 3/7*(0-4/7)) = (12/49, -12/49)
    x = np.zeros((1, 2))
    Wr = np.zeros((2, 4))
    idx = np.array([[3, 2]], dtype=np.int32)
    w = np.array([[4 / 7, 3 / 7]])
    dl, _, _ = O.route_bwd(x, Wr, idx, w, np.array([[1.0, 0.0]]))
    np.testing.assert_allclose(dl, [[0, 0, -12 / 49, 12 / 49]], rtol=1e-15, atol=0)


def test_gate_backward_invariants_and_loops():
    rng = np.random.default_rng(5)
    T, d, E, k = 9, 5, 6, 3
    x = rng.normal(size=(T, d))
    Wr = rng.normal(size=(d, E))
    idx, w = O.route_topk(O.route_logits(x, Wr), k)
    dw = rng.normal(size=(T, k))
    dl, dWr, dxg = O.route_bwd(x, Wr, idx, w, dw)
    np.testing.assert_allclose(dl.sum(1), 0.0, atol=1e-15)
    for t in range(T):
        for e in range(E):
            if e not in idx[t]:
                assert dl[t, e] == 0.0
    ref_dWr = np.zeros((d, E))
    ref_dx = np.zeros((T, d))
    for t in range(T):
        for i in range(d):
            for e in range(E):
                ref_dWr[i, e] += x[t, i] * dl[t, e]
                ref_dx[t, i] += dl[t, e] * Wr[i, e]
    np.testing.assert_allclose(dWr, ref_dWr, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(dxg, ref_dx, rtol=1e-13, atol=1e-14)


def test_activation_identities():
    a = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(O.gelu(a) - O.gelu(-a), a, atol=1e-15)
    np.testing.assert_allclose(O.silu(a) - O.silu(-a), a, atol=1e-15)
    assert O.gelu(np.array(0.0)) == 0.0 and O.gelu_grad(np.array(0.0)) == 0.5
    assert O.silu_grad(np.array(0.0)) == 0.5
    # against the standard library's erf / erfc, element by element
    for v in a:
        phi = 0.5 * math.erfc(-v / math.sqrt(2.0))
        assert O.gelu(np.array(v)) == pytest.approx(v * phi, rel=1e-13, abs=1e-16)
    # Phi by Simpson integration of the normal density from -12 (independent of any erf routine)
    for v in (-3.0, -0.7, 0.3, 1.9, 4.0):
        n = 20000
        g = np.linspace(-12.0, v, n + 1)
        pdf = np.exp(-0.5 * g * g) / math.sqrt(2 * math.pi)
        cdf = (g[1] - g[0]) / 3 * (pdf[0] + pdf[-1] + 4 * pdf[1:-1:2].sum() + 2 * pdf[2:-1:2].sum())
        assert O.gelu(np.array(v)) == pytest.approx(v * cdf, rel=1e-10)
    # the tanh approximation is NOT what is computed (it differs by ~1e-3 near |a|~2)
    tanh_form = 0.5 * a * (1 + np.tanh(math.sqrt(2 / math.pi) * (a + 0.044715 * a ** 3)))
    assert np.abs(tanh_form - O.gelu(a)).max() > 1e-4
    # derivatives by central differences
    h = 1e-6
    np.testing.assert_allclose((O.gelu(a + h) - O.gelu(a - h)) / (2 * h), O.gelu_grad(a), atol=1e-8)
    np.testing.assert_allclose((O.silu(a + h) - O.silu(a - h)) / (2 * h), O.silu_grad(a), atol=1e-8)


def test_golden_gate_closed_forms():
    import os
    from fractions import Fraction
    path = os.path.join(os.path.dirname(__file__), "golden", "gate_closed_forms.txt")
    n = 0
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        k, vals, ids, ws = [p.strip() for p in line.split(";")]
        logits = np.log(np.array([[float(v) for v in vals.split()]]))
        idx, w = O.route_topk(logits, int(k))
        assert idx[0].tolist() == [int(v) for v in ids.split()]
        np.testing.assert_allclose(w[0], [float(Fraction(v)) for v in ws.split()], rtol=1e-14)
        n += 1
    assert n == 5
