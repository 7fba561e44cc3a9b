"""The library's host planner against the oracle (Section 4.2, Algorithm 1).  Host-only calls: no GPU needed."""
import random

import pytest

from oracle import asymea_oracle as A
from paper_2504_03871_amd import binding as B

GROUPS = [(1, 1), (1, 2), (2, 1), (2, 4), (4, 2), (1, 4), (8, 2), (3, 9)]


def both(n, L, M, N, ta, t_attn, t_exp, n_min=None, n_max=None):
    want = A.plan(n, L, M, N, ta, t_attn, t_exp, n_min, n_max)
    got = B.moe_asymea_plan(n, L, M, N, ta, t_attn, t_exp, 0 if n_min is None else n_min,
                            -1 if n_max is None else n_max)
    return want, got


def test_figure_example():
    assert B.moe_asymea_plan(6, 3, 1, 1, 3.0, 3.0, 4.0) == [0, 1, 1]


def test_unbounded_matches_oracle_exactly():
    rnd = random.Random(3)
    for _ in range(2000):
        M, N = rnd.choice(GROUPS)
        n = N * rnd.randint(1, 8)
        L = rnd.randint(1, 64)
        ta = rnd.uniform(0.1, 5.0)
        t_exp = ta + rnd.uniform(-0.5, 6.0)
        t_attn = rnd.uniform(0.05, 5.0)
        want, got = both(n, L, M, N, ta, t_attn, t_exp)
        assert want == got, (n, L, M, N, ta, t_attn, t_exp)


def test_unbounded_matches_the_exact_cumulative_form():
    """The library against the oracle's second form (exact rationals, floors of cumulative quotients), which is
    not a copy of the listing; inputs whose quotients sit within 1e-9 of an integer are skipped."""
    rnd = random.Random(13)
    checked = 0
    for _ in range(2000):
        M, N = rnd.choice(GROUPS)
        n, L = N * rnd.randint(1, 8), rnd.randint(1, 64)
        ta = rnd.uniform(0.1, 5.0)
        t_exp, t_attn = ta + rnd.uniform(-0.5, 6.0), rnd.uniform(0.05, 5.0)
        want, margin = A.plan_exact(n, L, M, N, ta, t_attn, t_exp)
        if margin < 1e-9:
            continue
        checked += 1
        assert B.moe_asymea_plan(n, L, M, N, ta, t_attn, t_exp) == want, (n, L, M, N, ta, t_attn, t_exp)
    assert checked > 1900


def test_bounded_matches_oracle_exactly():
    rnd = random.Random(4)
    for _ in range(2000):
        M, N = rnd.choice(GROUPS)
        n = N * rnd.randint(1, 8)
        L = rnd.randint(1, 64)
        ta = rnd.uniform(0.1, 5.0)
        t_exp = ta + rnd.uniform(0.001, 6.0)
        t_attn = rnd.uniform(0.05, 5.0)
        n_min = rnd.randint(0, 40)
        n_max = n_min + rnd.randint(0, 60)
        want, got = both(n, L, M, N, ta, t_attn, t_exp, n_min, n_max)
        assert want == got, (n, L, M, N, ta, t_attn, t_exp, n_min, n_max)


def test_errors():
    bad = [dict(n=0), dict(L=0), dict(M=2, N=3), dict(M=0), dict(t_attn=-30.0), dict(ta=float("nan")),
           dict(n_min=5, n_max=4), dict(ta=9.0, n_min=2, n_max=8)]
    ok = dict(n=8, L=4, M=1, N=1, ta=1.0, t_attn=1.0, t_exp=2.0, n_min=0, n_max=-1)
    for b in bad:
        a = {**ok, **b}
        with pytest.raises(B.MoeError) as ei:
            B.moe_asymea_plan(a["n"], a["L"], a["M"], a["N"], a["ta"], a["t_attn"], a["t_exp"], a["n_min"], a["n_max"])
        assert ei.value.code == -2, b
    # no bubble, no lower bound: zeros
    assert B.moe_asymea_plan(8, 3, 1, 1, 2.0, 1.0, 2.0) == [0, 0, 0]


def test_shares_match_oracle_owner_and_partition():
    for n, M, N in ((8, 1, 1), (8, 2, 4), (8, 4, 2), (12, 1, 4), (16, 8, 2), (32, 2, 2)):
        _, n_2 = A.chunk_sizes(M, N)
        for o_l in range(0, n // N + 1, n_2):
            own = A.expert_owner(n, M, N, o_l)
            cover = [0] * n
            for role, cnt, tag in ((0, N, 'exp'), (1, M, 'attn')):
                for r in range(cnt):
                    lo, hi = B.moe_asymea_shares(n, M, N, o_l, role, r)
                    for e in range(n):
                        mine = own[e] == (tag, r)
                        assert lo[e] == 0 and hi[e] == (2 ** 31 - 1 if mine else 0)
                        cover[e] += hi[e] > 0
            assert cover == [1] * n
    for args in ((8, 4, 2, 1, 0, 0), (8, 1, 1, 9, 0, 0), (8, 1, 1, 1, 2, 0), (8, 2, 4, 1, 0, 4), (8, 2, 4, 1, 1, 2),
                 (9, 1, 2, 1, 0, 0)):
        with pytest.raises(B.MoeError) as ei:
            B.moe_asymea_shares(*args)
        assert ei.value.code == -2, args
