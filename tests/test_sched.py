"""Scheduling rules (Section 6.1) and the bottleneck-free range (eq. (9)): the oracle against
what the paper prints and states, and the C library against the oracle.  CPU only."""
import heapq
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import sched_oracle as O
from paper_2602_21548_amd import sched as S
import paper_2602_21548_amd as K


# --------------------------------------------------------------------------
# eq. (9)
# --------------------------------------------------------------------------

def test_pd_range_worked_example_from_the_paper():
    # Section 4.2: g = 8, s = 1, M ~ 500 GB/s, Bs ~ 50 GB/s  ->  1/7 <= P/D <= 7/2
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "pd_range_example.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert rows
    for g, s, M, Bs, ln, ld, hn, hd in (map(int, r) for r in rows):
        r = O.pd_range(g, s, M, Bs)
        assert Fraction(r["lo"]).limit_denominator(100) == Fraction(ln, ld)
        assert Fraction(r["hi"]).limit_denominator(100) == Fraction(hn, hd)
        assert r["feasible"]
    r = O.pd_range(8, 1, 500, 50)
    assert r["hi_de_read"] == 6 and r["hi_de_write"] == 3.5 and r["hi_dram"] == 3.5


@pytest.mark.parametrize("g,s,M,Bs", [(8, 1, 500, 50), (8, 2, 800, 100), (4, 1, 300, 25), (16, 3, 1000, 150)])
def test_pd_range_bounds_follow_from_the_traffic_sums(g, s, M, Bs):
    """Re-derive each bound from eqs. (1)-(8): at the bound the link is exactly full."""
    r = O.pd_range(g, s, M, Bs)
    B = Bs / s

    def traffic(P, D):
        Tp, Tc = Bs / (D * g * g), Bs / (P * g * g)       # per pair, PE read path / DE read path
        return dict(pe_write=(Tp + Tc) * D * g, de_read=(Tp + 2 * Tc) * P * g, de_write=(2 * Tp + Tc) * P * g,
                    de_mem=(3 + 2 * P / D) * Bs)
    D = 1000.0
    assert traffic(r["lo"] * D, D)["pe_write"] == pytest.approx(B)
    assert traffic(r["hi_de_read"] * D, D)["de_read"] == pytest.approx(B)
    assert traffic(r["hi_de_write"] * D, D)["de_write"] == pytest.approx(B)
    assert traffic(r["hi_dram"] * D, D)["de_mem"] == pytest.approx(M)
    # inside the range nothing is over its limit
    if r["feasible"]:
        mid = (r["lo"] + r["hi"]) / 2
        t = traffic(mid * D, D)
        assert t["pe_write"] <= B * (1 + 1e-9) and t["de_read"] <= B * (1 + 1e-9)
        assert t["de_write"] <= B * (1 + 1e-9) and t["de_mem"] <= M * (1 + 1e-9)


@pytest.mark.parametrize("g,s,M,Bs", [(8, 1, 500, 50), (8, 2, 800, 100), (8, 3, 500, 150), (4, 1, 100, 25)])
def test_pd_range_library_matches_oracle(g, s, M, Bs):
    want, got = O.pd_range(g, s, M, Bs), S.kvl_pd_range(g, s, M, Bs)
    for k in want:
        assert got[k] == pytest.approx(want[k], rel=1e-15), k
    with pytest.raises(K.KvlError):
        S.kvl_pd_range(8, 8, 500, 50)


# --------------------------------------------------------------------------
# Algorithm 1
# --------------------------------------------------------------------------

def _pe_case(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    n = int(rng.integers(1, 9))
    beta = int(rng.integers(50_000, 400_000))
    alpha = int(rng.integers(10_000, 200_000))
    tok = rng.integers(0, int(beta * 1.5), size=n).tolist()
    node = rng.integers(0, max(1, n // 2 + 1), size=n)
    node_q = rng.integers(0, alpha * 2, size=node.max() + 1)
    read_q = node_q[node].tolist()                                # engines of a node report the same queue
    Q = rng.integers(1_000, 70_000, size=int(rng.integers(0, 30))).tolist()
    return tok, read_q, Q, alpha, beta


# Cases worked by hand from the text of Section 6.1 ("PE Scheduling"): an engine is overloaded once its
# unfinished tokens exceed beta, overloaded engines get nothing, engines on nodes with a short reading
# queue (<= alpha) come first, each request goes to the smallest tok of its category, tok is updated
# after every assignment, and the fetch ends when no engine is left.  (tok, read_q, Q, alpha, beta,
# expected assignment, expected tok)
PE_HAND_CASES = [
    # one engine, beta crossed by the second request: the third stays in the queue
    ([0], [0], [60, 60, 60], 5, 100, [0, 0, -1], [120]),
    # an engine at exactly beta is not overloaded: it takes one more request and no further one
    ([100], [0], [1, 1], 5, 100, [0, -1], [101]),
    # the short-queue engine fills up with the first request; the long-queue engine takes over
    # until it is over the limit too; the rest is returned
    ([90, 0], [0, 9], [20, 30, 30, 50, 50, 10], 5, 100, [0, 1, 1, 1, -1, -1], [110, 110]),
    # two short-queue engines: smallest tok at each step (60 vs 50 -> engine 1), both end over the limit
    ([0, 50], [1, 1], [60, 60, 60, 60], 5, 100, [0, 1, 0, -1], [120, 110]),
    # three engines, engine 0 overloaded from the start; engine 2 has the short queue and stays under beta
    ([150, 10, 40], [0, 9, 1], [5, 5, 5], 5, 100, [2, 2, 2], [150, 10, 55]),
    # no short queue: the long-queue engines share the load, smallest tok first
    ([150, 10, 40], [9, 9, 9], [20, 20, 20], 5, 100, [1, 1, 2], [150, 50, 60]),
    # everyone overloaded: nothing is assigned
    ([101, 200], [0, 0], [1, 2], 5, 100, [-1, -1], [101, 200]),
    # a request larger than beta still goes to an engine that is not overloaded
    ([0, 0], [0, 0], [500, 10, 10], 5, 100, [0, 1, 1], [500, 20]),
    # the short-queue engine is preferred even though the long-queue one is emptier
    ([80, 0], [0, 9], [10, 5], 5, 100, [0, 0], [95, 0]),
    # an engine that lands exactly on beta may take one more request
    ([40], [0], [60, 1, 1], 5, 100, [0, 0, -1], [101]),
    # a reading queue of exactly alpha counts as short
    ([50, 0], [5, 9], [10], 5, 100, [0], [60, 0]),
    # empty queue, no engines
    ([10], [0], [], 5, 100, [], [10]),
    ([], [], [7], 5, 100, [-1], []),
]


@pytest.mark.parametrize("case", PE_HAND_CASES, ids=[str(i) for i in range(len(PE_HAND_CASES))])
def test_pe_fetch_hand_cases(case):
    tok0, read_q, Q, alpha, beta, want, want_tok = case
    tok = list(tok0)
    assert O.pe_fetch(tok, read_q, Q, alpha, beta) == want
    assert tok == want_tok


@pytest.mark.parametrize("E,size,beta,n", [(1, 10, 100, 30), (3, 10, 95, 50), (4, 7, 100, 10), (8, 33_000, 600_000, 1024),
                                           (5, 100, 99, 20), (2, 1, 0, 5)])
def test_pe_fetch_closed_form_equal_engines_equal_requests(E, size, beta, n):
    """Idle engines of one category and requests of one size: an engine is eligible while
    k * size <= beta, so each takes floor(beta / size) + 1 requests, dealt round robin."""
    per_engine = beta // size + 1
    k = min(n, E * per_engine)
    tok = [0] * E
    got = O.pe_fetch(tok, [0] * E, [size] * n, alpha=1, beta=beta)
    assert got == [i % E for i in range(k)] + [-1] * (n - k)
    assert sum(tok) == k * size and max(tok) - min(tok) <= size
    if k < n:
        assert all(t == per_engine * size for t in tok)


@pytest.mark.parametrize("seed", range(10))
def test_pe_fetch_without_limits_is_greedy_list_scheduling(seed):
    """beta and alpha out of reach: Algorithm 1 is the textbook greedy that gives each job to the
    least loaded machine (a heap of loads)."""
    rng = np.random.Generator(np.random.PCG64(900 + seed))
    n = int(rng.integers(1, 9))
    tok0 = rng.integers(0, 100_000, size=n).tolist()
    Q = rng.integers(1, 70_000, size=40).tolist()
    heap = [(t, e) for e, t in enumerate(tok0)]
    heapq.heapify(heap)
    want = []
    for job in Q:
        t, e = heapq.heappop(heap)
        want.append(e)
        heapq.heappush(heap, (t + job, e))
    assert O.pe_fetch(list(tok0), [0] * n, Q, alpha=10**12, beta=10**15) == want


def _check_fetch_against_the_text(tok0, read_q, Q, alpha, beta, got, tok_after):
    """Replay a finished fetch and hold every step against the sentences of Section 6.1."""
    n = len(tok0)
    t = list(tok0)
    k = sum(a >= 0 for a in got)
    assert got[:k] == [a for a in got if a >= 0]                   # FIFO: a prefix of the queue is assigned
    for a, tokens_r in zip(got[:k], Q):
        assert t[a] <= beta                                        # never to an overloaded engine
        short = [e for e in range(n) if t[e] <= beta and read_q[e] <= alpha]
        long_ = [e for e in range(n) if t[e] <= beta and read_q[e] > alpha]
        cls = short if short else long_                            # short queues first
        assert a in cls and t[a] == min(t[e] for e in cls)         # the minimum of its category at that moment
        assert a == min(e for e in cls if t[e] == t[a])            # ties: lowest index
        t[a] += tokens_r
    if k < len(Q):
        assert all(x > beta for x in t)                            # the fetch ended because no engine was left
    assert t == tok_after and sum(t) == sum(tok0) + sum(Q[:k])     # tokens conserved


def _two_heap_simulation(tok0, read_q, Q, alpha, beta):
    """Different structure from the oracle's loop: one heap per queue class; an engine that is over
    the limit when it comes up is dropped for good."""
    heaps = ([(t, e) for e, t in enumerate(tok0) if read_q[e] <= alpha],
             [(t, e) for e, t in enumerate(tok0) if read_q[e] > alpha])
    for h in heaps:
        heapq.heapify(h)
    out = []
    for tokens_r in Q:
        for h in heaps:
            while h and h[0][0] > beta:
                heapq.heappop(h)
        h = heaps[0] if heaps[0] else heaps[1]
        if not h:
            break
        t, e = heapq.heappop(h)
        out.append(e)
        heapq.heappush(h, (t + tokens_r, e))
    return out + [-1] * (len(Q) - len(out))


@pytest.mark.parametrize("seed", range(40))
def test_pe_fetch_invariants(seed):
    tok0, read_q, Q, alpha, beta = _pe_case(seed)
    tok = list(tok0)
    got = O.pe_fetch(tok, read_q, Q, alpha, beta)
    _check_fetch_against_the_text(tok0, read_q, Q, alpha, beta, got, tok)
    assert got == _two_heap_simulation(tok0, read_q, Q, alpha, beta)


def test_pe_fetch_random_cases_do_end_part_way():
    """The random cases above must exercise the case that decides the reading."""
    part_way = 0
    for seed in range(40):
        tok0, read_q, Q, alpha, beta = _pe_case(seed)
        got = O.pe_fetch(list(tok0), read_q, Q, alpha, beta)
        k = sum(a >= 0 for a in got)
        part_way += 0 < k < len(Q)
    assert part_way >= 5


PE_MUTANTS = [
    ("categories frozen before the loop", "        if tok[pe] > beta:", "        if False:"),
    ("overloaded at beta already", "        if tok[pe] > beta:", "        if tok[pe] >= beta:"),
    ("initial classification off by one", "C1 = [e for e in G_PE if tok[e] > beta]\n    C2 = [e for e in G_PE if read_q[e] <= alpha and tok[e] <= beta]",
     "C1 = [e for e in G_PE if tok[e] >= beta]\n    C2 = [e for e in G_PE if read_q[e] <= alpha and tok[e] < beta]"),
    ("long queues first", "        if C2:\n            C = C2\n        elif C3:\n            C = C3", "        if C3:\n            C = C3\n        elif C2:\n            C = C2"),
    ("short queue means below alpha", "read_q[e] <= alpha and", "read_q[e] < alpha and"),
    ("largest tok", "pe = min(C, key=lambda e: (tok[e], e))", "pe = max(C, key=lambda e: (tok[e], -e))"),
    ("tok not updated", "tok[pe] = tok[pe] + tokens_r", "tok[pe] = tok[pe]"),
    ("no fallback once the short queues are full", "        elif C3:", "        elif C3 and not C1:"),
]


def _pe_battery(fetch):
    for tok0, read_q, Q, alpha, beta, want, want_tok in PE_HAND_CASES:
        tok = list(tok0)
        if fetch(tok, read_q, Q, alpha, beta) != want or tok != want_tok:
            return 1
    for seed in range(40):
        tok0, read_q, Q, alpha, beta = _pe_case(seed)
        tok = list(tok0)
        got = fetch(tok, read_q, Q, alpha, beta)
        try:
            _check_fetch_against_the_text(tok0, read_q, Q, alpha, beta, got, tok)
        except AssertionError:
            return 1
    return 0


@pytest.mark.parametrize("name,old,new", PE_MUTANTS, ids=[m[0] for m in PE_MUTANTS])
def test_planted_mistake_in_algorithm_1_is_caught(name, old, new):
    src = open(O.__file__).read()
    assert src.count(old) >= 1, "mutation pattern no longer matches the oracle source"
    scope = {"__name__": "sched_oracle_mutant"}
    exec(compile(src.replace(old, new), "sched_oracle_mutant.py", "exec"), scope)
    assert _pe_battery(O.pe_fetch) == 0                            # the battery passes on the oracle as it is
    try:
        rc = _pe_battery(scope["pe_fetch"])
    except (ValueError, IndexError, AssertionError):
        rc = 1
    assert rc != 0, f"no pin noticed: {name}"


@pytest.mark.parametrize("case", PE_HAND_CASES, ids=[str(i) for i in range(len(PE_HAND_CASES))])
def test_pe_fetch_library_hand_cases(case):
    tok0, read_q, Q, alpha, beta, want, want_tok = case
    got, tok = S.kvl_sched_pe_fetch(tok0, read_q, Q, alpha, beta)
    assert got == want and tok.tolist() == want_tok


@pytest.mark.parametrize("seed", range(40))
def test_pe_fetch_library_matches_oracle(seed):
    tok0, read_q, Q, alpha, beta = _pe_case(seed)
    tok = list(tok0)
    want = O.pe_fetch(tok, read_q, Q, alpha, beta)
    lib_assign, lib_tok = S.kvl_sched_pe_fetch(tok0, read_q, Q, alpha, beta)
    assert lib_assign == want and lib_tok.tolist() == tok


# --------------------------------------------------------------------------
# decode side
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(20))
def test_de_groups(seed):
    rng = np.random.Generator(np.random.PCG64(100 + seed))
    g0 = rng.integers(0, 500_000, size=int(rng.integers(1, 7))).tolist()
    Q = rng.integers(1_000, 70_000, size=int(rng.integers(0, 40))).tolist()
    g = list(g0)
    got = O.de_groups(g, Q)
    assert sum(g) == sum(g0) + sum(Q)
    # each request went to a group that was a minimum at that moment
    h = list(g0)
    for a, len_r in zip(got, Q):
        assert h[a] == min(h)
        h[a] += len_r
    lib, lib_g = S.kvl_sched_de_groups(g0, Q)
    assert lib == got and lib_g.tolist() == g


@pytest.mark.parametrize("seed", range(40))
def test_de_fetch_invariants_and_library(seed):
    rng = np.random.Generator(np.random.PCG64(200 + seed))
    n = int(rng.integers(1, 9))
    tok0 = rng.integers(0, 300_000, size=n).tolist()
    seq0 = rng.integers(0, 40, size=n).tolist()
    free0 = rng.integers(0, 200_000, size=n).tolist()
    Q = rng.integers(1_000, 90_000, size=int(rng.integers(0, 25))).tolist()
    tok, seq, free = list(tok0), list(seq0), list(free0)
    got, Z = O.de_fetch(tok, seq, free, Q)
    # Z is the stated formula over the fragmentation-free prefix R
    used, R = 0, []
    for len_r in Q:
        if used + len_r > sum(free0):
            break
        used += len_r
        R.append(len_r)
    assert Z == pytest.approx(1.05 * (sum(R) + sum(tok0)) / n)
    k = sum(a >= 0 for a in got)
    assert got[:k] == [a for a in got if a >= 0] and k <= len(R)      # a prefix, bounded by |R|
    # replay: every choice fits, prefers the under-threshold class by seq, else min tok
    t, s, f = list(tok0), list(seq0), list(free0)
    for a, len_r in zip(got[:k], Q):
        fits = [e for e in range(n) if f[e] >= len_r]
        assert a in fits
        under = [e for e in fits if t[e] + len_r <= Z]
        if under:
            assert a in under and s[a] == min(s[e] for e in under)
        else:
            assert t[a] == min(t[e] for e in fits)
        t[a] += len_r; s[a] += 1; f[a] -= len_r
    if k < len(Q):
        assert all(f[e] < Q[k] for e in range(n))                     # the fetch ended for lack of HBM
    assert (t, s, f) == (tok, seq, free) and all(x >= 0 for x in f)
    lib, lib_z, lt, ls, lf = S.kvl_sched_de_fetch(tok0, seq0, free0, Q)
    assert lib == got and lib_z == pytest.approx(Z, rel=1e-15)
    assert (lt.tolist(), ls.tolist(), lf.tolist()) == (tok, seq, free)


# Cases worked by hand from Section 6.1 ("DE Scheduling Phase 2"): R is the head of the queue that fits the group's
# free HBM taken as one piece; Z = 1.05 (sum of R's lengths + sum of tok) / |E|; among the engines with room for the
# request those with tok + len <= Z come first and the one with the fewest requests is taken, otherwise the one with
# the smallest tok; the fetch ends at the first request no engine has room for.
# (tok, seq, free_hbm, Q, expected assignment, expected Z)
DE_HAND_CASES = [
    # engine 0 would go over Z = 78.75, so the request goes to engine 1 although that one holds more requests
    ([100, 0], [1, 5], [1000, 1000], [50], [1], 78.75),
    # both over Z = 126: the smaller tok wins
    ([100, 90], [1, 5], [1000, 1000], [50], [1], 126.0),
    # the group's free HBM as one piece would hold the request (so it is in R), but no engine does: the fetch ends
    ([0, 0], [0, 0], [40, 45], [50], [-1], 26.25),
    # a lone request on idle engines is over Z = 3.5 everywhere: smallest tok, lowest index
    ([0, 0, 0], [3, 1, 2], [100, 100, 100], [10], [0], 3.5),
    # six equal requests, Z = 21: fewest requests first, an engine drops to the other class once it holds two
    ([0, 0, 0], [3, 1, 2], [100, 100, 100], [10] * 6, [1, 1, 2, 0, 2, 0], 21.0),
    # R holds three requests (60 tokens free in all) but fragmentation lets only two in
    ([0, 0], [0, 0], [30, 30], [20, 20, 20, 20], [0, 1, -1, -1], 31.5),
    # Z = 89.25: under-threshold first (engine 1, then 0), then both over and the smaller tok
    ([50, 0], [0, 9], [100, 100], [60, 30, 30], [1, 0, 1], 89.25),
    # only engine 1 has room for the first request; it is over Z but the only choice
    ([10, 10], [2, 2], [15, 100], [20, 5], [1, 0], 23.625),
    # engine 1 lands exactly on Z = 35: that is not over it, and it has fewer requests than engine 0
    ([5, 15, 60], [9, 1, 0], [100, 100, 100], [20], [1], 35.0),
]


@pytest.mark.parametrize("case", DE_HAND_CASES, ids=[str(i) for i in range(len(DE_HAND_CASES))])
def test_de_fetch_hand_cases(case):
    tok0, seq0, free0, Q, want, want_z = case
    tok, seq, free = list(tok0), list(seq0), list(free0)
    got, Z = O.de_fetch(tok, seq, free, Q)
    assert got == want and Z == pytest.approx(want_z, rel=1e-12)
    placed = [(e, n) for e, n in zip(got, Q) if e >= 0]
    assert sum(tok) == sum(tok0) + sum(n for _, n in placed) and sum(free) == sum(free0) - sum(n for _, n in placed)
    lib, lib_z, lt, ls, lf = S.kvl_sched_de_fetch(tok0, seq0, free0, Q)
    assert lib == want and lib_z == pytest.approx(want_z, rel=1e-12)
    assert (lt.tolist(), ls.tolist(), lf.tolist()) == (tok, seq, free)


DE_MUTANTS = [
    ("threshold factor 1.5", "Z = 1.05 * (sum(R) + sum(tok)) / len(tok)", "Z = 1.5 * (sum(R) + sum(tok)) / len(tok)"),
    ("Z ignores the queued requests", "Z = 1.05 * (sum(R) + sum(tok)) / len(tok)", "Z = 1.05 * sum(tok) / len(tok)"),
    ("R is the whole queue", "        if used + len_r > total_free:\n            break", "        if False:\n            break"),
    ("at Z counts as over", "high = [e for e in fits if tok[e] + len_r > Z]\n        rest = [e for e in fits if not tok[e] + len_r > Z]",
     "high = [e for e in fits if tok[e] + len_r >= Z]\n        rest = [e for e in fits if not tok[e] + len_r >= Z]"),
    ("under-threshold class by tok", "de = min(rest, key=lambda e: (seq[e], e))", "de = min(rest, key=lambda e: (tok[e], e))"),
    ("over-threshold class by seq", "de = min(high, key=lambda e: (tok[e], e))", "de = min(high, key=lambda e: (seq[e], e))"),
    ("over-threshold engines first", "        if rest:\n            de = min(rest", "        if not high:\n            de = min(rest"),
    ("room is not checked", "fits = [e for e in E if free_hbm[e] >= len_r]", "fits = [e for e in E]"),
    ("free HBM not reduced", "        free_hbm[de] -= len_r", "        free_hbm[de] -= 0"),
    ("request count not updated", "        seq[de] += 1", "        seq[de] += 0"),
]


def _de_battery(fetch):
    for tok0, seq0, free0, Q, want, want_z in DE_HAND_CASES:
        got, Z = fetch(list(tok0), list(seq0), list(free0), Q)
        if got != want or abs(Z - want_z) > 1e-9:
            return 1
    return 0


@pytest.mark.parametrize("name,old,new", DE_MUTANTS, ids=[m[0] for m in DE_MUTANTS])
def test_planted_mistake_in_decode_phase_2_is_caught(name, old, new):
    src = open(O.__file__).read()
    assert src.count(old) >= 1, "mutation pattern no longer matches the oracle source"
    scope = {"__name__": "sched_oracle_mutant"}
    exec(compile(src.replace(old, new), "sched_oracle_mutant.py", "exec"), scope)
    assert _de_battery(O.de_fetch) == 0
    try:
        rc = _de_battery(scope["de_fetch"])
    except (ValueError, IndexError, AssertionError, ZeroDivisionError):
        rc = 1
    assert rc != 0, f"no hand case noticed: {name}"


def test_read_side():
    for a, b in ((0, 0), (5, 9), (9, 5), (7, 7)):
        want = O.read_side(a, b)
        assert want == (1 if b < a else 0)
        assert S.kvl_sched_read_side(a, b) == want


# --------------------------------------------------------------------------
# the rules driven by a request stream of the published shape
# --------------------------------------------------------------------------

def test_trace_driven_replay_library_follows_the_oracle():
    """Requests of the 64K agent trace arrive in waves; prefill engines fetch with Algorithm 1,
    decode groups and engines with the two decode phases; work drains between waves.  At every
    step the library decides as the oracle does, and load stays balanced."""
    import kvl_workloads as W
    t = W.agent_trace(64, n_traj=120)
    rng = np.random.Generator(np.random.PCG64(4242))
    order = rng.permutation(t.traj.size)[:6000]
    lens = (t.context + t.append)[order].tolist()                 # tokens(r): the request's total length
    n_pe, n_groups, per_group = 8, 2, 4
    alpha, beta = 150_000, 200_000
    pe_tok, pe_read = [0] * n_pe, [0] * n_pe
    g_tok = [0] * n_groups
    de_tok = [[0] * per_group for _ in range(n_groups)]
    de_seq = [[0] * per_group for _ in range(n_groups)]
    de_free = [[3_000_000] * per_group for _ in range(n_groups)]
    pos, steps, part_way, waiting = 0, 0, 0, []
    while pos < len(lens) or waiting:
        arrived = lens[pos:pos + int(rng.integers(1, 40))]
        pos += len(arrived)
        wave = waiting + arrived                                  # requests a fetch left behind keep their place
        # prefill side
        o_tok = list(pe_tok)
        want = O.pe_fetch(o_tok, pe_read, wave, alpha, beta)
        got, l_tok = S.kvl_sched_pe_fetch(pe_tok, pe_read, wave, alpha, beta)
        assert got == want and l_tok.tolist() == o_tok
        placed = [(e, n) for e, n in zip(want, wave) if e >= 0]
        waiting = wave[len(placed):]
        part_way += 0 < len(placed) < len(wave)
        assert all(e < 0 for e in want[len(placed):])
        pe_tok = o_tok
        for e, n in placed:                                       # reads queue on the engine's node (2 engines per node)
            pe_read[e] += n
            pe_read[e ^ 1] = pe_read[e]
        # decode side: groups, then engines inside each group
        done = [n for _, n in placed]
        og = list(g_tok)
        want_g = O.de_groups(og, done)
        got_g, lg = S.kvl_sched_de_groups(g_tok, done)
        assert got_g == want_g and lg.tolist() == og
        g_tok = og
        for g in range(n_groups):
            q = [n for n, gg in zip(done, want_g) if gg == g]
            ot, os_, of = list(de_tok[g]), list(de_seq[g]), list(de_free[g])
            want_d, z = O.de_fetch(ot, os_, of, q)
            got_d, lz, lt, ls, lf = S.kvl_sched_de_fetch(de_tok[g], de_seq[g], de_free[g], q)
            assert got_d == want_d and lz == pytest.approx(z, rel=1e-15)
            assert (lt.tolist(), ls.tolist(), lf.tolist()) == (ot, os_, of)
            de_tok[g], de_seq[g], de_free[g] = ot, os_, of
        # drain: engines work off a share of what they hold
        for e in range(n_pe):
            d = int(pe_tok[e] * rng.uniform(0.2, 0.9))
            pe_tok[e] -= d
            pe_read[e] = int(pe_read[e] * rng.uniform(0.1, 0.8))
        for e in range(0, n_pe, 2):
            pe_read[e + 1] = pe_read[e]
        for g in range(n_groups):
            for e in range(per_group):
                d = int(de_tok[g][e] * rng.uniform(0.3, 0.9))
                de_tok[g][e] -= d
                de_free[g][e] += d
                de_seq[g][e] = int(de_seq[g][e] * 0.5)
            g_tok[g] = sum(de_tok[g])
        steps += 1
    assert steps > 100
    assert part_way > 10                                          # fetches did end for lack of an engine under beta
