"""CPU timeline model of zebra parallelism.  TEST INFRASTRUCTURE ONLY.

A plain event-driven simulation of the execution model of Section 4.1 of the paper: tasks A (attention
computation), E (expert computation), D (dispatch all-to-all) and C (combine all-to-all), forward and
backward, for layer i and micro-batch j; a task starts once the task it depends on has finished AND
every earlier task of its stream has finished (the paper's two constraints: data dependency, and one
task at a time per stream).  It exists to check the task order the library's engine uses against the
paper's Theorem 1, and may be imported only by the tests.

Model (readings of the paper):
  * The model has L attention blocks with an expert block between consecutive ones: A_1 E_1 A_2 ...
    E_{L-1} A_L.  That is what makes Theorem 1's attention order put A^F_{L,j} directly before A^B_{L,j}
    and its expert order run over layers 1 .. L-1.
  * Streams: the attention GPUs' compute stream (all A tasks), the expert GPUs' compute stream (all E
    tasks), and two communication streams, one per direction (attention->expert carries D^F and, in the
    backward pass, the gradient of the combine; expert->attention carries C^F and the gradient of the
    dispatch).  Communication tasks are served first come, first served, in the order in which the
    tasks they depend on finish (the closing remark of Theorem 1).
  * Durations are per task kind; every GPU of a kind behaves alike, so one stream per kind suffices.

Asymmetric expert assignment (Section 4.2): `simulate_forward_asymea` adds the tasks of a layer whose expert GPUs
have given o of their n experts to the attention GPUs.  Readings: the attention GPUs compute a layer's offloaded
experts for every micro-batch AFTER that layer's attention of all micro-batches (the paper's sentence on the
figure), each such task needs the dispatch of its micro-batch (tokens arrive from the other attention GPUs), the
combine of a micro-batch waits for both parts, and the expert GPUs' task shrinks to (n - o) / n of its time.
The figure's numbers (60 % fewer bubbles, 10 % faster, 6 % bubbles on the expert GPUs) depend on the time one
expert takes on an attention GPU and on the communication times, which only the drawing holds: for those three
numbers, parity unpinned.  What the text fixes is pinned: with nothing offloaded the model is the default one,
a hand-computed timeline, the two scheduling constraints, and the two qualitative statements (offloading one of
six experts in the later layers shortens the forward pass and leaves the attention stream without bubbles after
the second layer's attention; offloading in the first layer too does not shorten it further and opens bubbles
on the expert GPUs).

Pins (tests/test_zebra_timeline.py): a hand-computed timeline, the steady-state share of time the
attention stream computes (T_A / T_E when experts are slower; the 75 % of the paper's Asym-EA figure
for experts a third slower), and brute force over every dependency-respecting order of a small problem
showing that none finishes earlier than the order of Theorem 1.
"""
from __future__ import annotations


def theorem1_attention_order(L, R):
    """(A^F_{1,1..R}) ... (A^F_{L-1,1..R}) (A^F_{L,1} A^B_{L,1} ... A^F_{L,R} A^B_{L,R}) (A^B_{L-1,1..R}) ... (A^B_{1,1..R})."""
    o = [("AF", i, j) for i in range(1, L) for j in range(1, R + 1)]
    for j in range(1, R + 1):
        o += [("AF", L, j), ("AB", L, j)]
    o += [("AB", i, j) for i in range(L - 1, 0, -1) for j in range(1, R + 1)]
    return o


def theorem1_expert_order(L, R):
    """(E^F_{1,1..R}) ... (E^F_{L-1,1..R}) (E^B_{L-1,1..R}) ... (E^B_{1,1..R})."""
    o = [("EF", i, j) for i in range(1, L) for j in range(1, R + 1)]
    o += [("EB", i, j) for i in range(L - 1, 0, -1) for j in range(1, R + 1)]
    return o


def dependencies(L, R):
    """task -> the one task it waits for (None for the first attention block)."""
    dep = {}
    for j in range(1, R + 1):
        dep[("AF", 1, j)] = None
        for i in range(1, L):
            dep[("DF", i, j)] = ("AF", i, j)
            dep[("EF", i, j)] = ("DF", i, j)
            dep[("CF", i, j)] = ("EF", i, j)
            dep[("AF", i + 1, j)] = ("CF", i, j)
        dep[("AB", L, j)] = ("AF", L, j)
        for i in range(L - 1, 0, -1):
            dep[("CB", i, j)] = ("AB", i + 1, j)     # gradient of the combine: attention -> expert
            dep[("EB", i, j)] = ("CB", i, j)
            dep[("DB", i, j)] = ("EB", i, j)         # gradient of the dispatch: expert -> attention
            dep[("AB", i, j)] = ("DB", i, j)
    return dep


STREAM_OF = {"AF": "attn", "AB": "attn", "EF": "exp", "EB": "exp", "DF": "a2e", "CB": "a2e", "CF": "e2a", "DB": "e2a"}


def simulate(L, R, dur, attn_order=None, exp_order=None):
    """Start and end time of every task.  `dur` maps a task kind ('AF', 'AB', 'EF', 'EB', 'DF', 'CF', 'CB',
    'DB') to its duration.  Returns (times: task -> (start, end), makespan); makespan is None when the given
    orders can never complete (a stream waits for a task that its own order puts later)."""
    attn_order = theorem1_attention_order(L, R) if attn_order is None else list(attn_order)
    exp_order = theorem1_expert_order(L, R) if exp_order is None else list(exp_order)
    dep = dependencies(L, R)
    assert sorted(attn_order) == sorted(t for t in dep if STREAM_OF[t[0]] == "attn")
    assert sorted(exp_order) == sorted(t for t in dep if STREAM_OF[t[0]] == "exp")
    times = {}
    free = {"attn": 0.0, "exp": 0.0, "a2e": 0.0, "e2a": 0.0}
    pos = {"attn": 0, "exp": 0}
    order = {"attn": attn_order, "exp": exp_order}
    waiting = {"a2e": [], "e2a": []}      # communication tasks whose producer has finished: (ready time, task)
    queued = set()
    n = len(dep)
    while len(times) < n:
        progressed = False
        # communication tasks become ready when the task they depend on is done
        for t, d in dep.items():
            s = STREAM_OF[t[0]]
            if s in waiting and t not in queued and d in times:
                waiting[s].append((times[d][1], t))
                queued.add(t)
        # candidates: the next task of each compute stream (if its dependency is done), the earliest-ready
        # task of each communication stream; run the one that can start first (ties: fixed stream order)
        cand = []
        for s in ("attn", "exp"):
            if pos[s] < len(order[s]):
                t = order[s][pos[s]]
                d = dep[t]
                if d is None or d in times:
                    cand.append((max(free[s], times[d][1] if d else 0.0), s, t))
        for s in ("a2e", "e2a"):
            if waiting[s]:
                ready, t = min(waiting[s])
                cand.append((max(free[s], ready), s, t))
        if cand:
            start, s, t = min(cand, key=lambda c: (c[0], c[1], c[2]))
            times[t] = (start, start + dur[t[0]])
            free[s] = start + dur[t[0]]
            if s in pos:
                pos[s] += 1
            else:
                waiting[s].remove(min(waiting[s]))
            progressed = True
        if not progressed:
            return times, None
    return times, max(e for _, e in times.values())


def chain_respecting_orders(chains):
    """Every interleaving of the given chains (lists) that keeps each chain's own order."""
    idx = [0] * len(chains)
    out = []
    total = sum(len(c) for c in chains)

    def rec():
        if len(out) == total:
            yield list(out)
            return
        for k, c in enumerate(chains):
            if idx[k] < len(c):
                out.append(c[idx[k]])
                idx[k] += 1
                yield from rec()
                idx[k] -= 1
                out.pop()

    yield from rec()


def attention_chains(L, R):
    return [[("AF", i, j) for i in range(1, L + 1)] + [("AB", i, j) for i in range(L, 0, -1)] for j in range(1, R + 1)]


def expert_chains(L, R):
    return [[("EF", i, j) for i in range(1, L)] + [("EB", i, j) for i in range(L - 1, 0, -1)] for j in range(1, R + 1)]


# ----------------------------------------------------------------------------- asymmetric expert assignment
def simulate_forward_asymea(L, R, t_a, t_e, n, offload, t_x, t_comm=0):
    """Forward pass of A_1 E_1 A_2 ... E_{L-1} A_L with R micro-batches when expert block i has offloaded
    offload[i-1] of its n experts to the attention GPUs.

    t_a: attention time per micro-batch; t_e: time of a whole expert block (n experts) on the expert GPUs per
    micro-batch; t_x: time of ONE offloaded expert on an attention GPU per micro-batch; t_comm: every
    all-to-all.  Tasks: AF (attention stream), EF (expert stream, duration t_e (n - o_i) / n), XF (attention
    stream: the offloaded experts of block i for micro-batch j, duration o_i t_x, placed after AF_{i,1..R}),
    DF and CF (communication streams, first come first served).  Use Fractions for exact times.
    Returns (times: task -> (start, end), makespan).
    """
    assert len(offload) == L - 1 and all(0 <= o <= n for o in offload)
    dep, dur, stream = {}, {}, {}
    for j in range(1, R + 1):
        dep[("AF", 1, j)] = []
        for i in range(1, L):
            o = offload[i - 1]
            dep[("DF", i, j)] = [("AF", i, j)]
            dep[("EF", i, j)] = [("DF", i, j)]
            dep[("CF", i, j)] = [("EF", i, j)]
            if o > 0:
                dep[("XF", i, j)] = [("DF", i, j)]
                dep[("CF", i, j)].append(("XF", i, j))
            dep[("AF", i + 1, j)] = [("CF", i, j)]
    for t in dep:
        k, i, _ = t
        stream[t] = {"AF": "attn", "XF": "attn", "EF": "exp", "DF": "a2e", "CF": "e2a"}[k]
        dur[t] = {"AF": t_a, "DF": t_comm, "CF": t_comm}.get(k)
        if k == "EF":
            dur[t] = t_e * (n - offload[i - 1]) / n
        if k == "XF":
            dur[t] = offload[i - 1] * t_x
    order = {"attn": asymea_attention_order(L, R, offload), "exp": [("EF", i, j) for i in range(1, L) for j in range(1, R + 1)]}
    pos = {"attn": 0, "exp": 0}
    free = {"attn": 0, "exp": 0, "a2e": 0, "e2a": 0}
    times = {}
    while len(times) < len(dep):
        cand = []
        for s in ("attn", "exp"):
            if pos[s] < len(order[s]):
                t = order[s][pos[s]]
                if all(d in times for d in dep[t]):
                    cand.append((max([free[s]] + [times[d][1] for d in dep[t]]), s, t))
        for t in dep:
            s = stream[t]
            if s in ("a2e", "e2a") and t not in times and all(d in times for d in dep[t]):
                ready = max(times[d][1] for d in dep[t])
                cand.append((max(free[s], ready), s, t))
        assert cand, "the given orders can never complete"
        # a communication stream serves the task that became ready first; ties and streams in a fixed order
        start, s, t = min(cand, key=lambda c: (c[0], c[1], c[2]))
        times[t] = (start, start + dur[t])
        free[s] = start + dur[t]
        if s in pos:
            pos[s] += 1
    return times, max(e for _, e in times.values())


def asymea_attention_order(L, R, offload):
    """Forward compute-stream order of an attention GPU: per layer the attention of every micro-batch, then (if
    the layer's expert block has offloaded experts) those experts for every micro-batch."""
    o = []
    for i in range(1, L + 1):
        o += [("AF", i, j) for j in range(1, R + 1)]
        if i < L and offload[i - 1] > 0:
            o += [("XF", i, j) for j in range(1, R + 1)]
    return o


def stream_bubbles(times, kinds, first=None, last=None):
    """Idle time of a stream between the start of task `first` and the end of task `last` (default: its first
    and last task): the span minus the time its tasks of the given kinds take."""
    iv = sorted(v for t, v in times.items() if t[0] in kinds)
    lo = iv[0][0] if first is None else times[first][0]
    hi = iv[-1][1] if last is None else times[last][1]
    busy = sum(min(e, hi) - max(s, lo) for s, e in iv if e > lo and s < hi)
    return (hi - lo) - busy
