"""CPU oracle for the asymmetric-expert-assignment planner.  TEST INFRASTRUCTURE ONLY.

Plain Python floats (IEEE double), the steps of the paper's Algorithm 1 ("gather and squeeze", Section
4.2) in the paper's order and notation, then the memory-bound variant of the same section (the
coefficients alpha and beta on the per-layer bubble).  It exists to check the host planner of the HIP
library and may be imported only by the tests; it shares no code with the library.

Inputs, in the paper's notation: n experts per layer, L layers, M attention GPUs and N expert GPUs in
a group, T_A_attn (attention module of one layer on an attention GPU), T_E_attn (one expert module on
an attention GPU), T_E_exp (a layer's expert module on an expert GPU), and optionally n_min / n_max, the
bounds on the total number of experts offloaded that the GPUs' memories impose.
Output: o[l], the number of experts each expert GPU offloads at layer l (0-based list of length L).

Readings where the paper is silent:
  * M must be a multiple of N or N a multiple of M (the paper's stated assumption): anything else is an
    error, as are non-positive n, L, M, N.
  * T_gather <= 0 (the expert GPUs are not the slower side): there is no bubble to gather, and the
    coefficients, which divide by T_gather, are undefined; the plan is all zeros.  A positive n_min is
    then an error (the lower bound cannot be met by this algorithm).
  * T_squeeze must be positive.
  * n_min / n_max = None: the unmodified Algorithm 1 (alpha = beta = 1).

Pins (tests/test_oracle_asymea.py): the worked example of the paper's Asym-EA figure (six experts, expert
GPUs a third slower, three layers: nothing offloaded at layer 1, one expert at layers 2 and 3),
hand-executed traces with exactly representable times, the closed form for the total number of chunks,
the clamps of the memory-bound variant, "alpha = 1 or beta = 1", and a brute-force re-statement of the
accumulate/subtract loop as "chunks so far = floor(l * T_gather / T_squeeze)" for exact inputs.
"""
from __future__ import annotations

import math


def chunk_sizes(M: int, N: int):
    """n_1 (experts one attention GPU acquires per chunk) and n_2 (experts one expert GPU offloads per
    chunk): Algorithm 1, first two lines."""
    if M <= 0 or N <= 0 or (M % N != 0 and N % M != 0):
        raise ValueError("M must be a multiple of N or N a multiple of M")
    n_1 = max(1, N // M)
    n_2 = n_1 * M // N
    assert n_1 * M == n_2 * N      # experts acquired by all attention GPUs == experts offloaded
    return n_1, n_2


def gather_squeeze_times(n, M, N, T_A_attn, T_E_attn, T_E_exp):
    """T_gather (bubble of one layer without offloading) and T_squeeze (bubble removed by offloading one
    chunk): Algorithm 1, lines three and four."""
    n_1, n_2 = chunk_sizes(M, N)
    T_gather = T_E_exp - T_A_attn
    T_squeeze = (T_E_exp * N / n) * n_1 + (T_E_attn * N / n) * n_2
    return T_gather, T_squeeze


def coefficients(n, L, M, N, T_A_attn, T_E_attn, T_E_exp, n_min, n_max):
    """alpha and beta of the memory-bound variant (Section 4.2, 'Addressing memory limitations')."""
    _, n_2 = chunk_sizes(M, N)
    T_gather, T_squeeze = gather_squeeze_times(n, M, N, T_A_attn, T_E_attn, T_E_exp)
    alpha = min((n_max // n_2) * T_squeeze / (L * T_gather), 1.0)
    beta = max(math.ceil(n_min / n_2) * T_squeeze / (L * T_gather), 1.0)
    return alpha, beta


def plan(n, L, M, N, T_A_attn, T_E_attn, T_E_exp, n_min=None, n_max=None):
    """Algorithm 1; with n_min / n_max given, its line that accumulates the bubble adds
    alpha * beta * T_gather instead of T_gather."""
    if n <= 0 or L <= 0:
        raise ValueError("n and L must be positive")
    n_1, n_2 = chunk_sizes(M, N)
    T_gather, T_squeeze = gather_squeeze_times(n, M, N, T_A_attn, T_E_attn, T_E_exp)
    if not T_squeeze > 0:
        raise ValueError("T_squeeze must be positive")
    bounded = n_min is not None or n_max is not None
    if bounded:
        n_min = 0 if n_min is None else n_min
        n_max = n * L if n_max is None else n_max
        if n_min < 0 or n_max < n_min:
            raise ValueError("need 0 <= n_min <= n_max")
    if T_gather <= 0:
        if bounded and n_min > 0:
            raise ValueError("no bubble to gather, yet a positive lower bound")
        return [0] * L
    step = T_gather
    if bounded:
        alpha, beta = coefficients(n, L, M, N, T_A_attn, T_E_attn, T_E_exp, n_min, n_max)
        step = alpha * beta * T_gather
    o = [0] * L
    t_bubble = 0.0
    for l in range(L):
        t_bubble = t_bubble + step
        if t_bubble >= T_squeeze:
            chunks = math.floor(t_bubble / T_squeeze)
            t_bubble = t_bubble - chunks * T_squeeze
            o[l] = chunks * n_2
    return o


def plan_exact(n, L, M, N, T_A_attn, T_E_attn, T_E_exp):
    """The unbounded plan in a second, independent form, in exact rational arithmetic on the given doubles.

    Algorithm 1's loop keeps t_bubble = l T_gather - (chunks so far) T_squeeze with 0 <= t_bubble < T_squeeze, so
    after layer l the chunks so far are floor(l T_gather / T_squeeze) and layer l offloads the difference of two
    consecutive floors.  No accumulation, no rounding: a misreading shared by the two double-precision copies of
    the listing (this module's `plan` and the library) would show against this form.  Also returns the smallest
    distance of any l T_gather / T_squeeze from an integer, so that a caller can tell inputs on which rounding
    could legitimately flip a floor."""
    from fractions import Fraction
    n_1, n_2 = chunk_sizes(M, N)
    ta, tx, te = Fraction(T_A_attn), Fraction(T_E_attn), Fraction(T_E_exp)
    T_gather = te - ta
    T_squeeze = te * N / n * n_1 + tx * N / n * n_2
    if T_gather <= 0:
        return [0] * L, Fraction(1)
    o, prev, margin = [], 0, Fraction(1)
    for l in range(1, L + 1):
        q = l * T_gather / T_squeeze
        c = q.numerator // q.denominator
        margin = min(margin, q - c, c + 1 - q)
        o.append((c - prev) * n_2)
        prev = c
    return o, margin


def expert_owner(n, M, N, o_l):
    """Which GPU computes each expert of a layer once every expert GPU has offloaded o_l experts.

    The paper says how many experts move, not which.  The reading used by the library: expert e lives
    on expert GPU e // (n/N); an expert GPU gives up the LAST o_l of its n/N experts; the offloaded
    experts, in ascending id, go to the attention GPUs in equal contiguous runs.  Returns a list of
    ('exp', g) / ('attn', a) per expert.
    """
    _, n_2 = chunk_sizes(M, N)
    if n % N != 0:
        raise ValueError("N must divide n")
    per = n // N
    if o_l < 0 or o_l > per or o_l % n_2 != 0:
        raise ValueError("o_l must be a multiple of n_2 in [0, n/N]")
    owner = [('exp', e // per) for e in range(n)]
    moved = [e for e in range(n) if e % per >= per - o_l]
    assert (len(moved) % M) == 0
    run = len(moved) // M
    for i, e in enumerate(moved):
        owner[e] = ('attn', i // run)
    return owner
