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


@pytest.mark.parametrize("seed", range(40))
def test_pe_fetch_invariants_and_library(seed):
    tok0, read_q, Q, alpha, beta = _pe_case(seed)
    tok = list(tok0)
    got = O.pe_fetch(tok, read_q, Q, alpha, beta)
    n = len(tok0)
    C2 = [e for e in range(n) if tok0[e] <= beta and read_q[e] <= alpha]
    C3 = [e for e in range(n) if tok0[e] <= beta and read_q[e] > alpha]
    allowed = C2 if C2 else C3
    if not allowed:
        assert got == [-1] * len(Q) and tok == tok0
    else:
        assert all(a in allowed for a in got)                     # overloaded never; short queues first
        # independent simulation: a heap of (tok, engine) over the allowed set
        heap = [(tok0[e], e) for e in allowed]
        heapq.heapify(heap)
        sim = []
        for tokens_r in Q:
            t, e = heapq.heappop(heap)
            sim.append(e)
            heapq.heappush(heap, (t + tokens_r, e))
        assert got == sim
        assert sum(tok) == sum(tok0) + sum(Q)                     # tokens conserved
    lib_assign, lib_tok = S.kvl_sched_pe_fetch(tok0, read_q, Q, alpha, beta)
    assert lib_assign == got and lib_tok.tolist() == tok


def test_pe_fetch_small_hand_cases():
    # three engines, beta = 100: engine 0 overloaded; engine 2 has the short queue
    assert O.pe_fetch([150, 10, 40], [0, 9, 1], [5, 5, 5], alpha=5, beta=100) == [2, 2, 2]
    # no short queue: the long-queue engines share the load, smallest tok first
    tok = [150, 10, 40]
    assert O.pe_fetch(tok, [9, 9, 9], [20, 20, 20], alpha=5, beta=100) == [1, 1, 2] and tok == [150, 50, 60]
    # everyone overloaded: nothing is assigned
    assert O.pe_fetch([101, 200], [0, 0], [1, 2], alpha=5, beta=100) == [-1, -1]


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
    alpha, beta = 150_000, 600_000
    pe_tok, pe_read = [0] * n_pe, [0] * n_pe
    g_tok = [0] * n_groups
    de_tok = [[0] * per_group for _ in range(n_groups)]
    de_seq = [[0] * per_group for _ in range(n_groups)]
    de_free = [[3_000_000] * per_group for _ in range(n_groups)]
    pos, steps = 0, 0
    while pos < len(lens):
        wave = lens[pos:pos + int(rng.integers(1, 40))]
        pos += len(wave)
        # prefill side
        o_tok = list(pe_tok)
        want = O.pe_fetch(o_tok, pe_read, wave, alpha, beta)
        got, l_tok = S.kvl_sched_pe_fetch(pe_tok, pe_read, wave, alpha, beta)
        assert got == want and l_tok.tolist() == o_tok
        placed = [(e, n) for e, n in zip(want, wave) if e >= 0]
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
