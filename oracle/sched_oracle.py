"""CPU oracle for the paper's scheduling rules (Section 6.1) and the
bottleneck-free P/D range (Section 4.2, eq. (9)).  TEST INFRASTRUCTURE ONLY.

Plain Python, in the paper's order and notation: sets C1, C2, C3 and the FIFO
loop of Algorithm 1; group sums for the first decode phase; the set R, the
threshold Z and the two categories of the second decode phase.

Pins (tests/test_sched.py): the range is pinned by the worked example the paper
prints (g = 8, s = 1, M ~ 500 GB/s, Bs ~ 50 GB/s gives 1/7 <= P/D <= 7/2) and by
re-deriving each bound from the traffic sums of eqs. (1)-(8).  The scheduling
rules are heuristics for which the paper prints no example.  Algorithm 1 is pinned
by cases worked by hand in which the limit beta is crossed in the middle of a fetch,
by a closed form (equal engines and equal requests: every engine takes
floor(beta / size) + 1 requests, in round-robin order), by the textbook special case
it reduces to without limits (greedy list scheduling onto the least loaded machine),
by a checker that replays a finished fetch against the sentences of the text, by a
two-heap simulation of different structure, and by mistakes planted in copies of this
file.  The second decode phase is pinned by hand-worked cases (the threshold Z, its two
categories, fragmentation against the set R, an engine exactly at Z), by the invariants the
text states, and by planted mistakes; the first phase by its arg-min invariant -- parity with
the paper's own implementation is unpinned (it prints no example).

Readings.  Algorithm 1: the three categories are defined by tok_e, and tok_e of the
chosen engine is updated after every assignment, so an engine whose unfinished tokens
have grown beyond beta is overloaded from then on and, like every overloaded engine,
gets nothing more in this fetch; that is what lets the
fetch end part-way and return the requests assigned so far, the case the text and the
listing both provide for inside the loop.  (With categories frozen before the loop
that case could only arise before the first request, and beta would bound nothing
within a fetch.)  An engine at exactly beta is not overloaded and may take one more
request.  Ties go to the lowest index; tokens(r) is the request's total length; phase
1 adds a request's length to its group's sum at once; HBM need and free HBM are
counted in tokens.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple


def pd_range(g: float, s: float, M: float, Bs: float) -> dict:
    """eq. (9) with its four ingredients (eqs. (3), (5), (7), (8))."""
    lo = s / (g - s)
    hi_de_read = (g - 2 * s) / s
    hi_de_write = (g - s) / (2 * s)
    hi_dram = (M / Bs - 3) / 2
    hi = min(hi_de_read, hi_de_write, hi_dram)
    return dict(lo=lo, hi=hi, hi_de_read=hi_de_read, hi_de_write=hi_de_write, hi_dram=hi_dram,
                feasible=lo <= hi)


def pe_fetch(tok: List[int], read_q: Sequence[int], Q: Sequence[int], alpha: int, beta: int) -> List[int]:
    """Algorithm 1.  tok is updated in place; returns the engine of each request of Q (-1: not assigned)."""
    G_PE = range(len(tok))
    C1 = [e for e in G_PE if tok[e] > beta]
    C2 = [e for e in G_PE if read_q[e] <= alpha and tok[e] <= beta]
    C3 = [e for e in G_PE if read_q[e] > alpha and tok[e] <= beta]
    assert sorted(C1 + C2 + C3) == list(G_PE)
    assigned = [-1] * len(Q)
    for i, tokens_r in enumerate(Q):               # FIFO
        if C2:
            C = C2
        elif C3:
            C = C3
        else:
            break                                  # terminate this fetch; assigned so far is returned
        pe = min(C, key=lambda e: (tok[e], e))
        assigned[i] = pe
        tok[pe] = tok[pe] + tokens_r
        if tok[pe] > beta:                         # the categories are defined by tok_e: pe is overloaded now
            C.remove(pe)
            C1.append(pe)
    return assigned


def de_groups(group_tok: List[int], Q: Sequence[int]) -> List[int]:
    """Decode phase 1: each request to the group with the smallest total tok."""
    out = []
    for len_r in Q:
        g = min(range(len(group_tok)), key=lambda k: (group_tok[k], k))
        out.append(g)
        group_tok[g] += len_r
    return out


def de_fetch(tok: List[int], seq: List[int], free_hbm: List[int], Q: Sequence[int]) -> Tuple[List[int], float]:
    """Decode phase 2 within one group.  Updates tok, seq, free_hbm; returns (assignment, Z)."""
    E = range(len(tok))
    total_free = sum(free_hbm)
    R = []
    used = 0
    for len_r in Q:                                # how many could be scheduled with no fragmentation
        if used + len_r > total_free:
            break
        used += len_r
        R.append(len_r)
    Z = 1.05 * (sum(R) + sum(tok)) / len(tok)
    assigned = [-1] * len(Q)
    for i, len_r in enumerate(Q):
        fits = [e for e in E if free_hbm[e] >= len_r]
        if not fits:
            break
        high = [e for e in fits if tok[e] + len_r > Z]
        rest = [e for e in fits if not tok[e] + len_r > Z]
        if rest:
            de = min(rest, key=lambda e: (seq[e], e))
        else:
            de = min(high, key=lambda e: (tok[e], e))
        assigned[i] = de
        tok[de] += len_r
        seq[de] += 1
        free_hbm[de] -= len_r
    return assigned, Z


def read_side(read_q_pe: int, read_q_de: int) -> int:
    """0: read on the prefill side, 1: on the decode side (the shorter queue; tie -> prefill)."""
    return 1 if read_q_de < read_q_pe else 0
