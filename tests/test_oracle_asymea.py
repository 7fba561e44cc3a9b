"""Pins for the planner oracle: Algorithm 1 and its memory-bound variant (Section 4.2 of the paper)."""
import math
import os
import random

import pytest

from oracle import asymea_oracle as A

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "asymea_figure_example.txt")


def test_figure_example_from_the_paper():
    rows = [l for l in open(GOLDEN).read().splitlines() if l and not l.startswith("#")]
    assert rows
    for row in rows:
        n, L, M, N, ta, te, tries, want = [f.strip() for f in row.split(";")]
        for t_e_attn in tries.split():
            got = A.plan(int(n), int(L), int(M), int(N), float(ta), float(t_e_attn), float(te))
            assert got == [int(v) for v in want.split()], (t_e_attn, got)
    # the same figure: attention GPUs compute 75 % of the time when experts are a third slower
    assert 3 / 4 == 0.75 and A.gather_squeeze_times(6, 1, 1, 3.0, 3.0, 4.0)[0] == 1.0


def test_chunk_sizes():
    # n_1 = max(1, N/M), n_2 = n_1 M / N, and what all attention GPUs acquire equals what all expert GPUs give
    assert A.chunk_sizes(1, 1) == (1, 1)
    assert A.chunk_sizes(2, 4) == (2, 1)
    assert A.chunk_sizes(4, 2) == (1, 2)
    assert A.chunk_sizes(3, 9) == (3, 1)
    assert A.chunk_sizes(8, 2) == (1, 4)
    for M, N in ((2, 3), (4, 6), (0, 1), (1, 0), (-2, 2)):
        with pytest.raises(ValueError):
            A.chunk_sizes(M, N)


def test_times_by_hand():
    # n=8, M=2, N=4: n_1=2, n_2=1.  T_squeeze = (8*4/8)*2 + (4*4/8)*1 = 8 + 2
    assert A.gather_squeeze_times(8, 2, 4, 6.0, 4.0, 8.0) == (2.0, 10.0)
    # M=4, N=2: n_1=1, n_2=2.  T_squeeze = (8*2/8)*1 + (4*2/8)*2 = 2 + 2; the two expert times are not
    # interchangeable here: swapped they would give (4*2/8)*1 + (8*2/8)*2 = 5
    assert A.gather_squeeze_times(8, 4, 2, 6.0, 4.0, 8.0) == (2.0, 4.0)


def test_hand_executed_traces():
    # bubble 2 per layer against a squeeze of 10: one chunk every fifth layer
    assert A.plan(8, 12, 2, 4, 6.0, 4.0, 8.0) == [0, 0, 0, 0, 1, 0, 0, 0, 0, 1, 0, 0]
    # several chunks per layer, remainder carried: T_gather=5, T_squeeze=6/4+2/4=2 -> 5:2 r1, 6:3 r0, ...
    assert A.plan(4, 5, 1, 1, 1.0, 2.0, 6.0) == [2, 3, 2, 3, 2]
    # n_2 = 2: every entry is a multiple of two.  T_gather=2, T_squeeze=4 -> a chunk every second layer
    assert A.plan(8, 6, 4, 2, 6.0, 4.0, 8.0) == [0, 2, 0, 2, 0, 2]
    # experts not slower than attention: nothing to gather
    assert A.plan(8, 4, 1, 1, 5.0, 1.0, 5.0) == [0, 0, 0, 0]
    assert A.plan(8, 4, 1, 1, 6.0, 1.0, 5.0) == [0, 0, 0, 0]


def test_cumulative_chunks_closed_form():
    """With integer times every step is exact, so after l layers floor(l T_gather / T_squeeze) chunks are out."""
    rnd = random.Random(5)
    for _ in range(300):
        M, N = rnd.choice([(1, 1), (1, 2), (2, 1), (2, 4), (4, 2), (1, 4), (8, 2)])
        n = N * rnd.randint(1, 4) * 4          # N/n * n_i stays a dyadic rational
        n_1, n_2 = A.chunk_sizes(M, N)
        L = rnd.randint(1, 40)
        t_a = float(rnd.randint(1, 20))
        t_exp = t_a + rnd.randint(1, 30)
        t_attn = float(rnd.randint(1, 30) * n)   # makes T_squeeze an integer
        t_exp = float(int(t_exp) * n)
        t_a = t_a * n
        tg, ts = A.gather_squeeze_times(n, M, N, t_a, t_attn, t_exp)
        assert tg == int(tg) and ts == int(ts)
        o = A.plan(n, L, M, N, t_a, t_attn, t_exp)
        run = 0
        for l in range(L):
            assert o[l] % n_2 == 0
            run += o[l] // n_2
            assert run == ((l + 1) * int(tg)) // int(ts)


def test_upper_bound_clamps_total():
    # natural plan: 8 layers * 4 / 2 = 16 chunks; memory allows floor(9 / 2) = 4 chunks of n_2 = 2 experts
    n, L, M, N = 8, 8, 4, 2
    ta, t_attn, t_exp = 4.0, 2.0, 8.0      # T_gather = 4, T_squeeze = (8*2/8)*1 + (2*2/8)*2 = 2 + 1
    tg, ts = A.gather_squeeze_times(n, M, N, ta, t_attn, t_exp)
    assert (tg, ts) == (4.0, 3.0)
    free = A.plan(n, L, M, N, ta, t_attn, t_exp)
    assert sum(free) // 2 == (8 * 4) // 3
    alpha, beta = A.coefficients(n, L, M, N, ta, t_attn, t_exp, 0, 9)
    assert beta == 1.0 and alpha == 4 * 3.0 / (8 * 4.0)
    o = A.plan(n, L, M, N, ta, t_attn, t_exp, n_min=0, n_max=9)
    # alpha * T_gather = 1.5 per layer: chunks land at layers 2, 4, 6, 8
    assert o == [0, 2, 0, 2, 0, 2, 0, 2] and sum(o) == (9 // 2) * 2


def test_lower_bound_raises_total():
    # natural plan: floor(8 * 1 / 4) = 2 chunks; the expert GPUs must shed at least 7 experts = 4 chunks of 2
    n, L, M, N = 8, 8, 4, 2
    ta, t_attn, t_exp = 7.0, 4.0, 8.0      # T_gather = 1, T_squeeze = (8*2/8)*1 + (4*2/8)*2 = 2 + 2
    assert A.gather_squeeze_times(n, M, N, ta, t_attn, t_exp) == (1.0, 4.0)
    assert sum(A.plan(n, L, M, N, ta, t_attn, t_exp)) == 2 * 2
    alpha, beta = A.coefficients(n, L, M, N, ta, t_attn, t_exp, 7, 64)
    assert alpha == 1.0 and beta == 4 * 4.0 / 8.0
    o = A.plan(n, L, M, N, ta, t_attn, t_exp, n_min=7, n_max=64)
    assert o == [0, 2, 0, 2, 0, 2, 0, 2] and sum(o) == math.ceil(7 / 2) * 2


def test_one_of_the_coefficients_is_one_and_total_within_bounds():
    rnd = random.Random(11)
    for _ in range(500):
        M, N = rnd.choice([(1, 1), (1, 2), (2, 1), (2, 4), (4, 2)])
        n_1, n_2 = A.chunk_sizes(M, N)
        n = N * rnd.randint(1, 8)
        L = rnd.randint(1, 48)
        ta = rnd.uniform(0.5, 4.0)
        t_exp = ta + rnd.uniform(0.01, 6.0)
        t_attn = rnd.uniform(0.2, 5.0)
        cmin = rnd.randint(0, 20)
        cmax = cmin + rnd.randint(0, 30)
        n_min = max(0, cmin * n_2 - rnd.randint(0, n_2 - 1))       # ceil(n_min / n_2) == cmin
        n_max = cmax * n_2 + rnd.randint(0, n_2 - 1)               # floor(n_max / n_2) == cmax
        alpha, beta = A.coefficients(n, L, M, N, ta, t_attn, t_exp, n_min, n_max)
        assert alpha == 1.0 or beta == 1.0
        o = A.plan(n, L, M, N, ta, t_attn, t_exp, n_min=n_min, n_max=n_max)
        assert all(v % n_2 == 0 and v >= 0 for v in o)
        chunks = sum(o) // n_2
        # the accumulated bubble L * step equals a whole number of squeezes only up to rounding, so the
        # floor may fall one short of the bound it aims at, never beyond the upper one
        assert chunks <= cmax
        assert chunks >= cmin - 1
        tg, ts = A.gather_squeeze_times(n, M, N, ta, t_attn, t_exp)
        natural = math.floor(L * tg / ts)
        if cmin <= natural <= cmax and alpha == 1.0 and beta == 1.0:
            assert abs(chunks - natural) <= 1


def test_argument_errors():
    with pytest.raises(ValueError):
        A.plan(0, 4, 1, 1, 1.0, 1.0, 2.0)
    with pytest.raises(ValueError):
        A.plan(8, 0, 1, 1, 1.0, 1.0, 2.0)
    with pytest.raises(ValueError):
        A.plan(8, 4, 2, 3, 1.0, 1.0, 2.0)
    with pytest.raises(ValueError):
        A.plan(8, 4, 1, 1, 1.0, -3.0, 2.0, )       # T_squeeze = 2/8 - 3/8 < 0
    with pytest.raises(ValueError):
        A.plan(8, 4, 1, 1, 3.0, 1.0, 2.0, n_min=2, n_max=4)   # no bubble, yet a lower bound
    with pytest.raises(ValueError):
        A.plan(8, 4, 1, 1, 1.0, 1.0, 2.0, n_min=5, n_max=4)


def test_expert_owner_partition():
    for n, M, N in ((8, 1, 1), (8, 2, 4), (8, 4, 2), (12, 1, 4), (16, 8, 2)):
        n_1, n_2 = A.chunk_sizes(M, N)
        per = n // N
        for o_l in range(0, per + 1, n_2):
            own = A.expert_owner(n, M, N, o_l)
            assert len(own) == n
            for g in range(N):
                assert sum(1 for w in own if w == ('exp', g)) == per - o_l
            for a in range(M):
                assert sum(1 for w in own if w == ('attn', a)) == o_l * N // M
            # an expert GPU keeps its first experts
            for e, w in enumerate(own):
                if e % per < per - o_l:
                    assert w == ('exp', e // per)
    with pytest.raises(ValueError):
        A.expert_owner(8, 4, 2, 1)      # not a multiple of n_2
    with pytest.raises(ValueError):
        A.expert_owner(8, 1, 1, 9)


def test_exact_cumulative_form_agrees_with_the_listing_and_the_figure():
    """`plan` (the listing's loop in doubles) against `plan_exact` (floors of exact cumulative quotients)."""
    import random
    assert A.plan_exact(6, 3, 1, 1, 3.0, 3.0, 4.0)[0] == [0, 1, 1]
    assert A.plan_exact(6, 4, 1, 1, 3.0, 3.0, 2.5)[0] == [0, 0, 0, 0]
    rnd = random.Random(11)
    checked = 0
    for _ in range(3000):
        M, N = rnd.choice([(1, 1), (1, 2), (2, 1), (2, 4), (4, 2), (3, 9)])
        n, L = N * rnd.randint(1, 8), rnd.randint(1, 48)
        ta = rnd.uniform(0.1, 5.0)
        te, tx = ta + rnd.uniform(-0.5, 6.0), rnd.uniform(0.05, 5.0)
        want, margin = A.plan_exact(n, L, M, N, ta, tx, te)
        if margin < 1e-9:        # a quotient this close to an integer: double rounding may flip its floor
            continue
        checked += 1
        assert A.plan(n, L, M, N, ta, tx, te) == want, (n, L, M, N, ta, tx, te)
    assert checked > 2900
