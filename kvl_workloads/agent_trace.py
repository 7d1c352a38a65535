"""Seeded multi-turn agent trajectories shaped like the paper's trace datasets.

The paper's three datasets (Section 7.1, table of agent trace statistics) are
private; what is published are five averages per dataset: interaction turns,
appended and generated tokens per turn, total tokens and context tokens.  This
module draws trajectories whose averages reproduce those five numbers, so that
the scheduling rules and the loader can be driven by request streams of the
published shape.  It only draws inputs; none of the method's arithmetic is here.

Model of one trajectory (a reading; the paper gives only the averages):
  final length  L  ~ normal around the published Total (sd 15 %), capped at MaxLen
  first prompt  P0 = f * L, with f chosen so that the mean context over the turns,
                about (P0 + L) / 2 for a context that grows evenly, is the published one
  turns         n  ~ lognormal with the published mean; its spread sigma is what makes
                the per-trajectory mean growth (L - P0) / n average to Append + Gen
                although (Total - P0) / Turns is much less (the statistics only fit
                together if they are means of per-trajectory means)
  per turn      the growth L - P0 is split over the turns with random weights, and each
                turn's growth into appended and generated tokens around the published ratio
Turn t of a trajectory is one request: its context so far is the cached (hit) prefix,
the appended tokens are the part prefill has to compute.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import BASE_SEED

# MaxLen (K tokens) -> published averages: turns, append, gen, total, context
PUBLISHED = {
    32: dict(turns=60, append=608, gen=148, total=28639, context=17183),
    48: dict(turns=106, append=474, gen=172, total=42607, context=25120),
    64: dict(turns=157, append=429, gen=176, total=55958, context=32721),
}


@dataclass
class AgentTrace:
    max_len: int                 # tokens
    traj: np.ndarray             # [n_requests] trajectory of each request
    turn: np.ndarray             # [n_requests] turn index inside its trajectory
    context: np.ndarray          # [n_requests] tokens already in the context = hit tokens of the request
    append: np.ndarray           # [n_requests] tokens appended this turn (to be prefilled)
    gen: np.ndarray              # [n_requests] tokens generated this turn
    n_traj: int

    def stats(self) -> dict:
        """The five averages, computed as the paper's fit together: per trajectory, then over trajectories."""
        first = np.flatnonzero(self.turn == 0)
        bounds = np.append(first, self.traj.size)
        turns, app, gen, ctx, total = [], [], [], [], []
        for a, b in zip(bounds[:-1], bounds[1:]):
            turns.append(b - a)
            app.append(self.append[a:b].mean())
            gen.append(self.gen[a:b].mean())
            ctx.append(self.context[a:b].mean())
            total.append(int(self.context[b - 1]) + int(self.append[b - 1]) + int(self.gen[b - 1]))
        return dict(turns=float(np.mean(turns)), append=float(np.mean(app)), gen=float(np.mean(gen)),
                    total=float(np.mean(total)), context=float(np.mean(ctx)),
                    hit_rate=float(self.context.sum() / (self.context.sum() + self.append.sum())))


def agent_trace(max_len_k: int = 64, n_traj: int = 500, seed: int = 0) -> AgentTrace:
    if max_len_k not in PUBLISHED:
        raise ValueError("max_len_k must be 32, 48 or 64")
    pub = PUBLISHED[max_len_k]
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 500 + max_len_k + 1000 * seed))
    max_len = max_len_k * 1024
    growth = pub["append"] + pub["gen"]
    f = 2.0 * pub["context"] / pub["total"] - 1.0                   # first prompt as a share of the final length
    # E[1/n] needed so that (1 - f) * Total * E[1/n] = Append + Gen; lognormal: E[n] E[1/n] = exp(sigma^2)
    sigma = float(np.sqrt(np.log(pub["turns"] * growth / ((1.0 - f) * pub["total"]))))
    mu = float(np.log(pub["turns"]) - sigma * sigma / 2.0)
    traj, turn, context, append, gen = [], [], [], [], []
    for i in range(n_traj):
        n = int(max(2, round(float(rng.lognormal(mu, sigma)))))
        # rounding may add a token per turn and part: keep the final length within MaxLen all the same
        L = float(np.clip(rng.normal(pub["total"], 0.15 * pub["total"]), 0.3 * pub["total"], max_len - 2 * n - 1))
        p0 = f * L
        w = rng.gamma(4.0, size=n)
        steps = (L - p0) * w / w.sum()                               # growth of each turn
        share = np.clip(rng.normal(pub["append"] / growth, 0.08, size=n), 0.05, 0.95)
        a = np.maximum(1, np.round(steps * share)).astype(np.int64)
        g = np.maximum(1, np.round(steps * (1.0 - share))).astype(np.int64)
        # the first turn's appended tokens are the first prompt itself; before it the context is empty
        ctx = np.empty(n, dtype=np.int64)
        ctx[0] = int(round(p0))
        ctx[1:] = ctx[0] + np.cumsum(a + g)[:-1]
        traj.append(np.full(n, i, dtype=np.int64))
        turn.append(np.arange(n, dtype=np.int64))
        context.append(ctx)
        append.append(a)
        gen.append(g)
    cat = np.concatenate
    return AgentTrace(max_len, cat(traj), cat(turn), cat(context), cat(append), cat(gen), n_traj)
