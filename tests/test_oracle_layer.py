"""Pins for the oracle's dispatch, expert FFN, combine and every gradient.

Brute force on tiny inputs, textbook special cases, round trips, additivity over complementary
shares, and central finite differences (Sections 2.1, 4.2 and 5 of the paper).
"""
import numpy as np
import pytest

from oracle import moe_oracle as O


# ----------------------------------------------------------------------------- permutation
def _brute_plan(idx, E, C):
    T, k = idx.shape
    counts = [0] * E
    kept = [0] * E
    offsets = [0] * (E + 1)
    lists = []
    for e in range(E):
        lst = []
        for t in range(T):
            for j in range(k):
                if idx[t, j] == e:
                    lst.append(t * k + j)
        counts[e] = len(lst)
        if C > 0:
            lst = lst[:C]
        kept[e] = len(lst)
        lists.append(lst)
    row_of = [-1] * (T * k)
    src_of = [-1] * (T * k)
    r = 0
    for e in range(E):
        offsets[e] = r
        for a in lists[e]:
            row_of[a] = r
            src_of[r] = a
            r += 1
    offsets[E] = r
    return counts, kept, offsets, row_of, src_of


@pytest.mark.parametrize("C", [0, 3, 7, 1000])
def test_plan_matches_brute_force(C):
    rng = np.random.default_rng(10 + C)
    for _ in range(60):
        E = int(rng.integers(1, 7))
        k = int(rng.integers(1, E + 1))
        T = int(rng.integers(1, 25))
        idx, _ = O.route_topk(rng.normal(size=(T, E)), k)
        got = O.dispatch_plan(idx, E, C)
        ref = _brute_plan(idx, E, C)
        for g, r in zip(got, ref):
            assert g.dtype == np.int32
            assert g.tolist() == r


def test_plan_invariants():
    rng = np.random.default_rng(11)
    T, E, k, C = 700, 8, 2, 150
    idx, _ = O.route_topk(rng.normal(size=(T, E)) - 0.4 * np.arange(E), k)
    counts, kept, offsets, row_of, src_of = O.dispatch_plan(idx, E, C)
    assert counts.sum() == T * k
    assert (kept == np.minimum(counts, C)).all()
    assert (offsets == np.concatenate([[0], np.cumsum(kept)])).all()
    live = row_of >= 0
    assert live.sum() == kept.sum() == offsets[E]
    assert (T * k - live.sum()) == np.maximum(counts - C, 0).sum() > 0
    assert len(set(row_of[live].tolist())) == live.sum()
    assert (src_of[row_of[live]] == np.nonzero(live)[0]).all()
    for e in range(E):
        seg = src_of[offsets[e]:offsets[e + 1]]
        assert (np.diff(seg) > 0).all()
        assert (idx.reshape(-1)[seg] == e).all()
    # the dropped ones are exactly the highest-token entries of each list
    for e in range(E):
        mine = np.nonzero(idx.reshape(-1) == e)[0]
        assert (row_of[mine[:kept[e]]] >= 0).all() and (row_of[mine[kept[e]:]] == -1).all()
    # unlimited capacity drops nothing
    assert (O.dispatch_plan(idx, E, 0)[3] >= 0).all()


def test_clamp_slices():
    kept = np.array([5, 0, 9])
    lo, hi = O.clamp_slices(kept)
    assert lo.tolist() == [0, 0, 0] and hi.tolist() == [5, 0, 9]
    lo, hi = O.clamp_slices(kept, [-3, 2, 4], [99, 1, 2])
    assert lo.tolist() == [0, 0, 4] and hi.tolist() == [5, 0, 4]      # hi<lo is empty


# ----------------------------------------------------------------------------- forward
def _setup(rng, T, d, f, E, k, act, gap=0.0):
    x = rng.normal(size=(T, d))
    Wr = rng.normal(size=(d, E)) / np.sqrt(d)
    W1 = rng.normal(size=(E, d, f)) * 0.3
    W1b = rng.normal(size=(E, d, f)) * 0.3 if act == O.ACT_SWIGLU else None
    W2 = rng.normal(size=(E, f, d)) * 0.3
    dout = rng.normal(size=(T, d))
    if gap > 0:
        # keep tokens whose k-th and (k+1)-th logits are well apart, so routing is locally constant
        l = np.sort(O.route_logits(x, Wr), axis=1)[:, ::-1]
        ok = np.ones(T, bool) if k == E else (l[:, k - 1] - l[:, k]) > gap
        ok &= (np.abs(np.diff(l[:, :k], axis=1)) > gap).all(axis=1) if k > 1 else True
        x, dout = x[ok], dout[ok]
    return x, Wr, W1, W1b, W2, dout


@pytest.mark.parametrize("act", [O.ACT_GELU, O.ACT_SWIGLU])
def test_single_expert_is_dense_ffn(act):
    rng = np.random.default_rng(20)
    T, d, f = 6, 4, 5
    x, Wr, W1, W1b, W2, dout = _setup(rng, T, d, f, 1, 1, act)
    r = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, 1, act)
    assert (r["w"] == 1.0).all() and r["row_of"].tolist() == list(range(T))
    ref = np.zeros((T, d))
    for t in range(T):
        h = np.zeros(f)
        for c in range(f):
            a = sum(x[t, i] * W1[0, i, c] for i in range(d))
            if act == O.ACT_GELU:
                h[c] = O.gelu(np.array(a))
            else:
                u = sum(x[t, i] * W1b[0, i, c] for i in range(d))
                h[c] = a / (1 + np.exp(-a)) * u
        for i in range(d):
            ref[t, i] = sum(h[c] * W2[0, c, i] for c in range(f))
    np.testing.assert_allclose(r["out"], ref, rtol=1e-12, atol=1e-14)


def test_forward_matches_token_loop():
    """out[t] = sum_j w_j * FFN_{e_j}(x[t]) computed token by token without any permutation."""
    rng = np.random.default_rng(21)
    T, d, f, E, k = 40, 6, 7, 5, 3
    for act in (O.ACT_GELU, O.ACT_SWIGLU):
        x, Wr, W1, W1b, W2, dout = _setup(rng, T, d, f, E, k, act)
        r = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, k, act)
        for t in range(T):
            acc = np.zeros(d)
            for j in range(k):
                e = r["idx"][t, j]
                a = x[t] @ W1[e]
                h = O.gelu(a) if act == O.ACT_GELU else O.silu(a) * (x[t] @ W1b[e])
                acc += r["w"][t, j] * (h @ W2[e])
            np.testing.assert_allclose(r["out"][t], acc, rtol=1e-12, atol=1e-14)


def test_zero_W2_and_linearity_in_W2():
    rng = np.random.default_rng(22)
    x, Wr, W1, W1b, W2, dout = _setup(rng, 30, 5, 6, 4, 2, O.ACT_GELU)
    r0 = O.moe_layer(x, Wr, None, W1, None, W2 * 0, dout, 2, O.ACT_GELU)
    assert (r0["out"] == 0).all()
    r1 = O.moe_layer(x, Wr, None, W1, None, W2, dout, 2, O.ACT_GELU)
    r3 = O.moe_layer(x, Wr, None, W1, None, W2 * 3, dout, 2, O.ACT_GELU)
    np.testing.assert_allclose(r3["out"], 3 * r1["out"], rtol=1e-13)


def test_identity_experts_round_trip():
    rng = np.random.default_rng(23)
    T, d, E, k = 200, 9, 6, 2
    x = rng.normal(size=(T, d))
    idx, w = O.route_topk(rng.normal(size=(T, E)), k)
    for C in (0, 40):
        counts, kept, offsets, row_of, src_of = O.dispatch_plan(idx, E, C)
        lo, hi = O.clamp_slices(kept)
        xp = O.dispatch_gather(x, src_of, offsets, lo, hi, k)
        assert not np.isnan(xp[:offsets[E]]).any()
        out = O.combine(xp, w, idx, row_of, offsets, lo, hi)
        keptw = (w * (row_of.reshape(T, k) >= 0)).sum(1, keepdims=True)
        if C == 0:
            np.testing.assert_allclose(keptw, 1.0, rtol=1e-14)
        else:
            assert (keptw < 0.999).any()
        np.testing.assert_allclose(out, x * keptw, rtol=1e-13, atol=1e-15)


# ----------------------------------------------------------------------------- shares (Section 4.2)
@pytest.mark.parametrize("act", [O.ACT_GELU, O.ACT_SWIGLU])
def test_complementary_shares_add_up(act):
    rng = np.random.default_rng(30)
    T, d, f, E, k = 120, 6, 5, 6, 2
    x, Wr, W1, W1b, W2, dout = _setup(rng, T, d, f, E, k, act)
    C = 30
    full = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, k, act, capacity=C)
    kept = full["kept"]
    cut = (kept * np.array([0.0, 0.3, 0.5, 1.0, 0.6, 0.2])).astype(int)
    a = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, k, act, capacity=C, lo=np.zeros(E, int), hi=cut)
    b = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, k, act, capacity=C, lo=cut, hi=kept)
    for name in ("out", "dx", "dW1", "dW2", "dWr", "dw", "dlogits") + (("dW1b",) if W1b is not None else ()):
        np.testing.assert_allclose(a[name] + b[name], full[name], rtol=1e-11, atol=1e-12, err_msg=name)
    # whole-expert split (the paper's asymmetric expert assignment): expert 0 has an empty share in
    # `a`, expert 3 a full one; the empty share contributes nothing and leaves its rows untouched
    assert (a["dW1"][0] == 0).all() and (a["dW2"][0] == 0).all()
    r0, r1 = full["offsets"][0], full["offsets"][1]
    assert np.isnan(a["x_perm"][r0:r1]).all() and np.isnan(a["fw"]["Y"][r0:r1]).all()
    np.testing.assert_allclose(a["dW1"][3], full["dW1"][3], rtol=1e-13)
    assert (b["dW1"][3] == 0).all()


# ----------------------------------------------------------------------------- finite differences
def _loss(x, Wr, W1, W1b, W2, dout, k, act, C, lo, hi):
    r = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, k, act, capacity=C, lo=lo, hi=hi)
    return (r["out"] * dout).sum()


@pytest.mark.parametrize("act", [O.ACT_GELU, O.ACT_SWIGLU])
@pytest.mark.parametrize("mode", ["full", "capacity", "partial"])
def test_gradients_by_central_differences(act, mode):
    rng = np.random.default_rng(40 + act)
    d, f, E, k = 5, 4, 4, 2
    x, Wr, W1, W1b, W2, dout = _setup(rng, 24, d, f, E, k, act, gap=2e-2)
    x, dout = x[:8], dout[:8]
    assert x.shape[0] == 8
    C = 3 if mode != "full" else 0
    base = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, k, act, capacity=C)
    lo = hi = None
    if mode == "partial":
        lo = base["kept"] // 3
        hi = base["kept"]
        hi[1] = lo[1]                                   # one expert with an empty share
    r = O.moe_layer(x, Wr, None, W1, W1b, W2, dout, k, act, capacity=C, lo=lo, hi=hi)
    if mode != "full":
        assert (r["row_of"] < 0).any()
    params = {"x": (x, r["dx"]), "Wr": (Wr, r["dWr"]), "W1": (W1, r["dW1"]), "W2": (W2, r["dW2"])}
    if W1b is not None:
        params["W1b"] = (W1b, r["dW1b"])
    h = 1e-6
    for name, (p, grad) in params.items():
        num = np.zeros_like(p)
        it = np.nditer(p, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = p[i]
            p[i] = old + h
            lp = _loss(x, Wr, W1, W1b, W2, dout, k, act, C, lo, hi)
            p[i] = old - h
            lm = _loss(x, Wr, W1, W1b, W2, dout, k, act, C, lo, hi)
            p[i] = old
            num[i] = (lp - lm) / (2 * h)
        scale = np.abs(grad).max()
        assert scale > 0
        np.testing.assert_allclose(grad, num, rtol=0, atol=2e-7 * max(scale, 1.0), err_msg=f"{name} {mode}")


def test_dw_is_gradient_of_weights():
    """dw is d(loss)/d(w) with w treated as free: check by perturbing w inside combine."""
    rng = np.random.default_rng(50)
    T, d, E, k = 12, 5, 4, 2
    y = rng.normal(size=(T * k, d))
    dout = rng.normal(size=(T, d))
    idx, w = O.route_topk(rng.normal(size=(T, E)), k)
    counts, kept, offsets, row_of, src_of = O.dispatch_plan(idx, E, 4)
    lo, hi = O.clamp_slices(kept)
    dy, dw = O.combine_bwd(dout, y, w, idx, row_of, offsets, lo, hi)
    h = 1e-6
    for t in range(T):
        for j in range(k):
            wp, wm = w.copy(), w.copy()
            wp[t, j] += h
            wm[t, j] -= h
            num = ((O.combine(y, wp, idx, row_of, offsets, lo, hi) -
                    O.combine(y, wm, idx, row_of, offsets, lo, hi)) * dout).sum() / (2 * h)
            assert dw[t, j] == pytest.approx(num, abs=1e-8)
            if row_of[t * k + j] < 0:
                assert dw[t, j] == 0.0
    live = row_of >= 0
    rows = row_of[live]
    tok = np.nonzero(live)[0] // k
    np.testing.assert_allclose(dy[rows], w.reshape(-1)[live][:, None] * dout[tok], rtol=1e-15)


def test_dot_scale_is_the_size_of_storage_rounding_in_d_topk_w():
    """The parity tests measure d_topk_w = <d_out, y_perm row> also against gpu_util.dot_scale.  Rounding y to
    fp16 (unit roundoff 2^-11, relative error uniform, variance u^2/3 at most) must move the dot product by about
    u/sqrt(3) times that scale, whatever the dot product itself cancels to."""
    from tests import gpu_util as U
    rng = np.random.default_rng(5)
    T, k, d = 400, 2, 128
    y = rng.standard_normal((T * k, d))
    d_out = rng.standard_normal((T, d))
    idx = np.zeros((T, k), dtype=np.int32)
    idx[:, 1] = 1
    # two experts: expert 0 holds the rows of slot 0, expert 1 those of slot 1
    order = np.argsort(idx.reshape(-1), kind="stable")
    row_of = np.empty(T * k, dtype=np.int64)
    row_of[order] = np.arange(T * k)
    offsets = np.array([0, T], dtype=np.int64)
    lo, hi = np.zeros(2, dtype=np.int64), np.array([T, T // 2], dtype=np.int64)            # half of expert 1 is foreign
    sc = U.dot_scale(d_out, y, idx, row_of, offsets, lo, hi)
    _, dw = O.combine_bwd(d_out, y, np.ones((T, k)), idx, row_of, offsets, lo, hi)
    _, dw16 = O.combine_bwd(d_out, y.astype(np.float16).astype(np.float64), np.ones((T, k)), idx, row_of, offsets, lo, hi)
    ok = O.in_share(idx, row_of, offsets, lo, hi).reshape(T, k)
    assert (sc[~ok] == 0).all() and (sc[ok] > 0).all()
    z = (dw16 - dw)[ok] / (2.0 ** -11 / np.sqrt(3) * sc[ok])
    assert 0.4 < z.std() < 1.0 and np.abs(z).max() < 5          # binade structure makes the variance a bit smaller
    # the scale is what the reference's own magnitude is when nothing cancels in particular
    assert 0.8 < np.sqrt((dw[ok] ** 2).mean()) / np.sqrt((sc[ok] ** 2).mean()) < 1.2
