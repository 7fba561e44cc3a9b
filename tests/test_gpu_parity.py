"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element.

Protocol for the gate (the top-k decision depends on fp32 rounding of x Wr): the GPU's logits are
compared with the oracle's fp64 logits within tolerance; the oracle's selection rule is then applied
to the GPU's own stored fp32 logits and must reproduce the GPU's indices bit for bit; every integer
output downstream is compared exactly.  Floating-point outputs: relative L2 error and max-abs error
relative to the largest reference magnitude, both <= 1e-5 (fp32) or 2e-2 (bf16 storage, fp32
accumulation).
"""
import numpy as np
import pytest

from paper_2504_03871_amd import synth as S
from tests import gpu_util as U

pytestmark = pytest.mark.gpu

W = S.WORKLOADS
CASES = {
    # the full fp32 configuration
    "cfg0": W["cfg0"],
    "cfg0_swiglu_partial_cap": W["cfg0"].scaled(act=S.ACT_SWIGLU, capacity_factor=0.9, partial=True, zipf_s=0.8),
    "f32_ragged": W["cfg0"].scaled(T=333, d=68, f=100, E=5, k=3, zipf_s=1.0),
    # reduced versions of the bf16 configurations: several row tiles per expert plus a ragged tail
    "cfg1_small": W["cfg1"].scaled(T=1000, d=256, f=512),
    "cfg2_small": W["cfg2"].scaled(T=2048, d=256, f=384),
    "cfg3_small": W["cfg3"].scaled(T=1536, d=512, f=448),
    "cfg4_small": W["cfg4"].scaled(T=2048, d=256, f=512),
    "cfg4z_small": W["cfg4z"].scaled(T=2048, d=256, f=512),
    "swiglu_partial_cap": W["cfg3"].scaled(T=1200, d=256, f=320, E=6, k=3, capacity_factor=0.8, partial=True, zipf_s=0.7),
    # degenerate shapes
    "one_expert": W["cfg1"].scaled(T=300, d=64, f=64, E=1, k=1),
    "k_equals_E": W["cfg1"].scaled(T=130, d=128, f=192, E=3, k=3),
    "one_token": W["cfg1"].scaled(T=1, d=64, f=128, E=4, k=2),
    "many_experts": W["cfg1"].scaled(T=700, d=128, f=128, E=200, k=8),
    # rows wider than one block of column groups, and not a power of two of them
    "wide_rows": W["cfg1"].scaled(T=150, d=4160, f=128, E=4, k=2),
    "d320_e16": W["cfg2"].scaled(T=900, d=320, f=256, E=16, k=2),
    # two and four expert tiles in the matrix-core gate kernel, a token count that is not a multiple of 32
    "e48_k4": W["cfg1"].scaled(T=333, d=192, f=128, E=48, k=4),
    "e100_k6": W["cfg1"].scaled(T=77, d=128, f=64, E=100, k=6),
    # the matrix-core gate weight gradient: a last column block of 64, a last K step of 11 tokens, three expert tiles
    "e40_d320": W["cfg1"].scaled(T=203, d=320, f=128, E=40, k=3),
    # d_ff long enough for split-K of the smallest row tiles: only such tiles / a full tile plus a small rest
    "split_k_tiny": W["cfg1"].scaled(T=40, d=128, f=2048, E=4, k=2),
    "split_k_mixed": W["cfg1"].scaled(T=620, d=128, f=2560, E=4, k=2),
    # fp16 storage (the paper trains in FP16 mixed precision, Section 6.1): the bf16 cases again
    "f16_cfg1_small": W["cfg1"].scaled(T=1000, d=256, f=512, dtype=S.DT_F16),
    "f16_cfg2_small": W["cfg2"].scaled(T=2048, d=256, f=384, dtype=S.DT_F16),
    "f16_cfg3_small": W["cfg3"].scaled(T=1536, d=512, f=448, dtype=S.DT_F16),
    "f16_cfg4z_small": W["cfg4z"].scaled(T=2048, d=256, f=512, dtype=S.DT_F16),
    "f16_swiglu_partial_cap": W["cfg3"].scaled(T=1200, d=256, f=320, E=6, k=3, capacity_factor=0.8, partial=True, zipf_s=0.7,
                                               dtype=S.DT_F16),
    "f16_many_experts": W["cfg1"].scaled(T=700, d=128, f=128, E=200, k=8, dtype=S.DT_F16),
    "f16_one_token": W["cfg1"].scaled(T=1, d=64, f=128, E=4, k=2, dtype=S.DT_F16),
    "f16_split_k_mixed": W["cfg1"].scaled(T=620, d=128, f=2560, E=4, k=2, dtype=S.DT_F16),
    # one token, two slots, both d_topk_w values a fifth of their uncancelled size
    "f16_one_token_cancelling": W["cfg1"].scaled(T=1, d=128, f=2560, E=64, k=2, dtype=S.DT_F16, zipf_s=0.8),
}


def run_case(w: S.Workload):
    import torch
    inp = S.make_inputs(w)
    L = U.make_layer(w, inp)
    tol = U.TOL[w.dtype]
    # shares need the kept counts: one index-only dispatch first, read back, then the real pass
    lo = hi = None
    if w.partial:
        L.route()
        L.dispatch(gather=False)
        torch.cuda.synchronize()
        lo, hi = S.partial_slices(w, U.host(L.kept))
        L.set_slices(lo, hi)
    U.fill_sentinels(L)
    L.forward()
    L.backward()
    torch.cuda.synchronize()

    g_logits = L.logits.cpu().numpy()
    ref = U.run_oracle(w, inp, gpu_logits=g_logits, lo=lo, hi=hi)
    rep = {}
    # (A) logits against the oracle's own fp64 logits
    rep["logits"] = U.assert_close("logits", g_logits.astype(np.float64), ref["logits"], tol)
    # (B) selection replayed by the oracle on the GPU's stored logits: bit-exact
    assert (U.host(L.topk_idx) == ref["idx"]).all(), "topk_idx"
    rep["topk_w"] = U.assert_close("topk_w", U.host(L.topk_w), ref["w"], 1e-5)
    # (C) tokens that the oracle's own fp64 logits would route differently must be near-ties
    own_idx, _ = U.O.route_topk(ref["logits"], w.k)
    diff = np.nonzero((own_idx != ref["idx"]).any(axis=1))[0]
    rep["routing_flips"] = len(diff)
    if len(diff) and w.k < w.E:
        # A flip needs two logits closer than the error of the GPU's two dot products.  With
        # S = max_e sum_i |x_i Wr_ie|: fp32 accumulation of d terms in some order leaves about
        # sqrt(d) * 2^-24 * S (random-walk estimate; the factor 8 is the margin); the bf16 and fp16 gates also
        # keep the weight as two bf16 terms, i.e. to 2^-17 relative, which adds 2^-17 * S per logit.
        acc = 8 * 2.0 ** -24 * np.sqrt(w.d)
        rep_w = 2 * 2.0 ** -17 if w.dtype != S.DT_F32 else 0.0    # fp32 inputs: plain fp32 FMAs on the fp32 weight
        mag = np.abs(inp["x"][diff].astype(np.float64)) @ np.abs(inp["Wr"].astype(np.float64))
        srt = np.sort(ref["logits"][diff], axis=1)[:, ::-1]
        gaps = np.abs(np.diff(srt[:, :w.k + 1], axis=1)).min(axis=1)
        assert (gaps <= (acc + rep_w) * mag.max(axis=1)).all(), "routing flip on a clear gap"
    # integer outputs: exact
    for name in ("counts", "kept", "offsets", "row_of", "src_of"):
        assert (U.host(getattr(L, name)) == ref[name]).all(), name
    # rows of the permuted buffers that belong to this GPU's shares
    A = w.T * w.k
    live = np.zeros(A, dtype=bool)
    for e in range(w.E):
        live[ref["offsets"][e] + ref["lo"][e]: ref["offsets"][e] + ref["hi"][e]] = True
    xp = U.host(L.x_perm)
    assert (xp[live] == ref["x_perm"][live]).all(), "x_perm rows differ"
    planes = ("A", "H") if w.act == S.ACT_GELU else ("G", "U", "H")
    for name, t in [("x_perm", L.x_perm), ("y_perm", L.y_perm), ("dy_perm", L.dy_perm), ("dx_perm", L.dx_perm)] + \
                   [("saved_" + p, L.saved_plane(i)) for i, p in enumerate(planes)]:
        assert U.untouched_rows(t, live), f"{name}: rows outside the shares were written"
    if live.any():
        for i, p in enumerate(planes):
            rep[p] = U.assert_close("saved " + p, U.host(L.saved_plane(i)), ref["fw"][p], tol)
        rep["y_perm"] = U.assert_close("y_perm", U.host(L.y_perm), ref["fw"]["Y"], tol)
        rep["dy_perm"] = U.assert_close("dy_perm", U.host(L.dy_perm), ref["dy_perm"], tol)
        rep["dx_perm"] = U.assert_close("dx_perm", U.host(L.dx_perm), ref["dx_perm"], tol)
    rep["out"] = U.assert_close("out", U.host(L.out), ref["out"], tol)
    # d_topk_w is a dot product over d_model that may cancel; with few slots every reference value can be such a
    # cancelled sum, so the uncancelled size of the sum is the second yardstick (see gpu_util.dot_scale)
    dw_scale = U.dot_scale(inp["d_out"], ref["fw"]["Y"], ref["idx"], ref["row_of"], ref["offsets"], ref["lo"], ref["hi"])
    rep["d_topk_w"] = U.assert_close("d_topk_w", U.host(L.d_topk_w), ref["dw"], tol, scale=dw_scale)
    dead = ~U.O.in_share(ref["idx"], ref["row_of"], ref["offsets"], ref["lo"], ref["hi"])
    assert (U.host(L.d_topk_w).reshape(-1)[dead] == 0).all(), "d_topk_w of dropped / foreign slots must be 0"
    rep["dW1"] = U.assert_close("dW1", U.host(L.dW1), ref["dW1"], tol)
    rep["dW2"] = U.assert_close("dW2", U.host(L.dW2), ref["dW2"], tol)
    if w.act == S.ACT_SWIGLU:
        rep["dW1b"] = U.assert_close("dW1b", U.host(L.dW1b), ref["dW1b"], tol)
    # gate backward, stage by stage: the oracle's softmax and linear backward applied to the GPU's own d_topk_w
    dl_s, dWr_s, dxg_s = U.O.route_bwd(inp["x"], inp["Wr"], ref["idx"], ref["w"], U.host(L.d_topk_w))
    rep["d_logits (stage)"] = U.assert_close("d_logits (stage)", U.host(L.d_logits), dl_s, tol)
    rep["dWr (stage)"] = U.assert_close("dWr (stage)", U.host(L.dWr), dWr_s, tol)
    rep["dx (stage)"] = U.assert_close("dx (stage)", U.host(L.dx), ref["dx_experts"] + dxg_s, tol)
    unsel = np.ones((w.T, w.E), bool)
    np.put_along_axis(unsel, ref["idx"].astype(np.int64), False, axis=1)
    assert (U.host(L.d_logits)[unsel] == 0).all()
    # and end to end against the oracle's own chain.  d_logits is w_j (dw_j - sum_i w_i dw_i): with a handful of
    # slots the difference can cancel what is left of already cancelled dot products, and then no fixed
    # tolerance relative to the reference holds, so this needs enough slots for the largest value to be typical
    if w.T * w.k >= 64:
        rep["d_logits"] = U.assert_close("d_logits", U.host(L.d_logits), ref["dlogits"], tol)
        rep["dWr"] = U.assert_close("dWr", U.host(L.dWr), ref["dWr"], tol)
        rep["dx"] = U.assert_close("dx", U.host(L.dx), ref["dx"], tol)
    return L, ref, rep


@pytest.mark.parametrize("name", list(CASES))
def test_parity(name):
    print(f"\n[case {name}] {CASES[name]}", flush=True)
    L, ref, rep = run_case(CASES[name])
    print({k: (f"{v[0]:.2e}", f"{v[1]:.2e}") if isinstance(v, tuple) else v for k, v in rep.items()}, flush=True)
    w = CASES[name]
    if w.capacity and w.zipf_s > 0:
        assert (ref["row_of"] < 0).any(), "this case is meant to drop tokens"


def test_determinism_and_accumulate():
    """Same inputs twice give the same bits; accumulate=1 adds to the weight gradients."""
    import torch
    w = CASES["cfg2_small"]
    inp = S.make_inputs(w)
    L = U.make_layer(w, inp)
    L.step()
    torch.cuda.synchronize()
    first = {n: getattr(L, n).clone() for n in ("out", "dx", "dW1", "dW2", "dWr", "row_of", "src_of", "d_topk_w")}
    U.fill_sentinels(L)
    L.step()
    torch.cuda.synchronize()
    for n, t in first.items():
        assert torch.equal(t, getattr(L, n)), n
    L.ffn_bwd(accumulate=1)
    torch.cuda.synchronize()
    for n in ("dW1", "dW2"):
        assert torch.equal(getattr(L, n), 2 * first[n]), n


def test_route_from_given_logits_with_ties():
    """Oracle logits in, GPU selection out: heavy ties, signed zeros, k up to 8, E up to 256."""
    import torch
    from paper_2504_03871_amd import binding as B
    rng = np.random.default_rng(7)
    for E, k, T in ((8, 2, 513), (64, 8, 100), (65, 3, 77), (256, 8, 50), (5, 5, 33)):
        vals = np.array([-1.5, -0.0, 0.0, 0.25, 3.0], dtype=np.float32)
        logits = vals[rng.integers(0, 5, size=(T, E))]
        logits[::3] = rng.normal(size=(len(logits[::3]), E)).astype(np.float32)
        cfg = B.make_cfg(T, 64, 64, E, k)
        dl = torch.from_numpy(logits).cuda()
        idx = torch.empty(T, k, dtype=torch.int32, device="cuda")
        wt = torch.empty(T, k, dtype=torch.float32, device="cuda")
        B.moe_route(cfg, None, None, None, dl, None, idx, wt)
        torch.cuda.synchronize()
        ridx, rw = U.O.route_topk(logits, k)
        assert (idx.cpu().numpy() == ridx).all(), (E, k)
        U.assert_close("w", wt.cpu().numpy().astype(np.float64), rw, 1e-5)
        assert np.allclose(wt.cpu().numpy().sum(1), 1.0, atol=1e-6)


def test_identity_round_trip_on_gpu():
    """dispatch followed by combine of the permuted input itself returns the input (bf16: within rounding)."""
    import torch
    w = CASES["cfg1_small"]
    inp = S.make_inputs(w)
    L = U.make_layer(w, inp)
    L.route()
    L.dispatch()
    L.y_perm.copy_(L.x_perm)
    L.combine()
    torch.cuda.synchronize()
    U.assert_close("round trip", U.host(L.out), inp["x"].astype(np.float64), 2 ** -8)


def test_empty_token_batch():
    import torch
    from paper_2504_03871_amd import binding as B
    cfg = B.make_cfg(0, 64, 64, 4, 2)
    i32 = dict(dtype=torch.int32, device="cuda")
    counts, kept, offsets = torch.full((4,), -1, **i32), torch.full((4,), -1, **i32), torch.full((5,), -1, **i32)
    dummy = torch.zeros(64, **i32)
    ws = torch.zeros(max(B.moe_workspace_bytes(cfg), 256), dtype=torch.uint8, device="cuda")
    B.moe_dispatch(cfg, None, dummy, None, None, counts, kept, offsets, dummy, dummy, None, ws)
    torch.cuda.synchronize()
    assert counts.tolist() == [0] * 4 and kept.tolist() == [0] * 4 and offsets.tolist() == [0] * 5


def test_gate_weight_gradient_on_a_second_stream():
    """The two halves of the gate backward (weight gradient; input gradient) run as separate calls, the
    first on a second stream next to the expert backward: same bits as the one-call, one-stream backward."""
    import torch
    for name in ("cfg2_small", "many_experts"):
        w = CASES[name]
        inp = S.make_inputs(w)
        L = U.make_layer(w, inp)
        L.step()
        torch.cuda.synchronize()
        names = ("dx", "dWr", "d_logits", "dW1", "dW2", "dx_perm")
        first = {n: getattr(L, n).clone() for n in names}
        U.fill_sentinels(L)
        L.enable_gate_overlap()
        L.step()
        L.step()        # events and the side buffers are reused
        torch.cuda.synchronize()
        for n in names:
            a, b = getattr(L, n), first[n]
            view = torch.int16 if a.element_size() == 2 else torch.int32
            assert torch.equal(a.view(view), b.view(view)), (name, n)
        assert torch.equal(L.side_d_logits, L.d_logits)


def test_dispatch_many_blocks_and_ids_out_of_range():
    """Index-only dispatch on assignment lists long enough for the scanned-prefix path (more than 64 blocks
    of 1024 assignments), with and without capacity, and with expert ids outside [0, E): those are dropped
    assignments (row_of = -1, not counted) and never index memory."""
    import torch
    from paper_2504_03871_amd import binding as B
    rng = np.random.default_rng(11)
    for T, k, E, cap, bad in ((40000, 2, 8, 0, False), (33000, 8, 200, 1500, False), (70001, 1, 16, 0, True),
                              (3000, 2, 8, 0, True)):
        idx = rng.integers(0, E, size=(T, k)).astype(np.int32)
        if bad:
            hit = rng.random(size=idx.shape) < 0.01
            idx[hit] = rng.choice(np.array([-1, -5, E, E + 7, 2 ** 30], dtype=np.int64), size=int(hit.sum())).astype(np.int32)
        cfg = B.make_cfg(T, 64, 64, E, k, capacity=cap)
        i32 = dict(dtype=torch.int32, device="cuda")
        counts, kept, offsets = torch.full((E,), -7, **i32), torch.full((E,), -7, **i32), torch.full((E + 1,), -7, **i32)
        row_of, src_of = torch.full((T * k,), -7, **i32), torch.full((T * k,), -7, **i32)
        ws = torch.empty(B.moe_workspace_bytes(cfg), dtype=torch.uint8, device="cuda")
        B.moe_dispatch(cfg, None, torch.from_numpy(idx).cuda(), None, None, counts, kept, offsets, row_of, src_of, None, ws)
        torch.cuda.synchronize()
        r = U.O.dispatch_plan(idx, E, cap)    # the oracle lists expert e's assignments by `flat == e`: other ids belong to no list
        for name, got, want in zip(("counts", "kept", "offsets", "row_of", "src_of"), (counts, kept, offsets, row_of, src_of), r):
            assert (got.cpu().numpy() == want).all(), (T, k, E, cap, bad, name)
        if bad:
            flat = idx.reshape(-1)
            assert (row_of.cpu().numpy()[(flat < 0) | (flat >= E)] == -1).all()


def test_random_workloads():
    """Thirty seeded random small workloads (all three storage types, both activations, 1 to 130 experts, ragged
    token counts, capacity, skew, partial shares, the split-K widths) through the same checks as the named cases."""
    import random
    rnd = random.Random(20250403871)
    for it in range(30):
        dt = rnd.choice([S.DT_BF16, S.DT_BF16, S.DT_F16, S.DT_F32])
        act = rnd.choice([S.ACT_GELU, S.ACT_SWIGLU])
        E = rnd.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 32, 33, 64, 70, 130])
        k = rnd.randint(1, min(E, 8))
        mult = 64 if dt != S.DT_F32 else 4
        d = mult * rnd.randint(1, 6 if dt != S.DT_F32 else 40)
        f = mult * rnd.randint(1, 9 if dt != S.DT_F32 else 60)
        if dt != S.DT_F32 and rnd.random() < 0.15:
            f = 2048 + 512 * rnd.randint(0, 2)                       # wide enough for split-K of the smallest tiles
        T = rnd.choice([1, 7, 33, 100, 257, 300, 511, 600, 1025, 1500])
        if dt == S.DT_F32:
            T = min(T, 300)
        base = W["cfg3"] if act == S.ACT_SWIGLU else W["cfg1"]
        w = base.scaled(T=T, d=d, f=f, E=E, k=k, capacity_factor=rnd.choice([0.0, 0.0, 0.7, 1.1]),
                        partial=rnd.random() < 0.4, zipf_s=rnd.choice([0.0, 0.8, 1.3]), dtype=dt)
        print(f"\n[random {it}] {w}", flush=True)
        run_case(w)


def test_random_wide_row_workloads():
    """Twelve more seeded random workloads with long token rows (1024 to 4096 elements, one of them not a multiple
    of 128) and 16-bit storage: the eight-wave gate kernels, the long-row forms of gather and combine, the last column
    block of the matrix-core gate weight gradient."""
    import random
    rnd = random.Random(3871)
    for it in range(12):
        dt = rnd.choice([S.DT_BF16, S.DT_F16])
        act = rnd.choice([S.ACT_GELU, S.ACT_SWIGLU])
        E = rnd.choice([2, 8, 16, 17, 40, 64, 130, 200])
        k = rnd.randint(1, min(E, 8))
        d = rnd.choice([1024, 2048, 2112, 4096])
        f = 64 * rnd.randint(1, 3)
        T = rnd.choice([1, 33, 257, 600, 1025])
        base = W["cfg3"] if act == S.ACT_SWIGLU else W["cfg1"]
        w = base.scaled(T=T, d=d, f=f, E=E, k=k, capacity_factor=rnd.choice([0.0, 0.0, 0.8]),
                        partial=rnd.random() < 0.4, zipf_s=rnd.choice([0.0, 1.0]), dtype=dt)
        print(f"\n[random wide {it}] {w}", flush=True)
        run_case(w)
