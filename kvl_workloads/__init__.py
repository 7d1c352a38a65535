"""Seeded synthetic inputs for the layer-wise KV-cache load path.

This module only *draws* inputs: request lengths, block tables and pool fills.
It holds none of the method's arithmetic (no offsets, no prefix sums, no
gather or scatter), so the CPU oracle and the HIP library can both be fed from
it without sharing anything else.

The shapes stand in for the paper's private agent traces: context lengths of
tens of thousands of tokens, a few hundred appended tokens per turn, hit rates
of 95 % and more (Section 3, Table 2), 64-token blocks (Section 4.1) and the
Layer-Block layout ``[1, tokens, bytes]`` (Appendix A.5).

Seeds: ``BASE_SEED + config index`` for lengths, ``+100`` for block tables,
``+200`` for pool fills (NumPy ``Generator(PCG64)``).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20260221

__all__ = [
    "BASE_SEED", "Layout", "Side", "Workload", "config", "tiny",
    "make_tables", "fill_pool", "fill_pool_fast", "random_payload",
    "sentinel_pool", "N_CONFIGS", "agent_trace", "AgentTrace", "PUBLISHED_TRACE_STATS", "from_trace",
]

N_CONFIGS = 5


@dataclass(frozen=True)
class Layout:
    """Geometry of one paged cache layer (Appendix A.5 Layer Block).

    ``row_bytes[p]`` is the cache bytes per token per layer of plane ``p``
    (one plane for MLA-style caches, two for separate K and V).
    """
    n_layers: int
    block_tokens: int
    row_bytes: Tuple[int, ...]

    @property
    def n_planes(self) -> int:
        return len(self.row_bytes)


@dataclass
class Side:
    """One engine's paged pool addressing: pool size and per-request tables."""
    pool_blocks: int
    tables: List[np.ndarray]  # int32, one per request


@dataclass
class Workload:
    name: str
    index: int
    layout: Layout
    hit: np.ndarray          # uint32 [R] cached-prefix tokens per request
    app: np.ndarray          # uint32 [R] appended (miss) tokens per request
    src: Side                # decode-side pool the hit KV is gathered from
    dst: Side                # prefill-side pool the hit KV is scattered into
    fill: str                # "bf16_uniform" or "bytes"
    seed: int
    notes: dict = field(default_factory=dict)

    @property
    def n_requests(self) -> int:
        return int(self.hit.shape[0])


# --------------------------------------------------------------------------
# block tables
# --------------------------------------------------------------------------

def _blocks_needed(hit: np.ndarray, app: np.ndarray, bs: int) -> np.ndarray:
    tot = hit.astype(np.int64) + app.astype(np.int64)
    return (tot + bs - 1) // bs


def _repair_adjacent(tbl: np.ndarray, rng: np.random.Generator) -> None:
    """In place: make sure no two consecutive entries are physically adjacent."""
    n = tbl.shape[0]
    if n < 4:
        return
    for _ in range(64):
        d = np.abs(np.diff(tbl.astype(np.int64)))
        bad = np.nonzero(d == 1)[0] + 1
        if bad.size == 0:
            return
        for i in bad:
            j = int(rng.integers(0, n))
            tbl[i], tbl[j] = tbl[j], tbl[i]
    raise RuntimeError("could not fragment table")


def make_tables(n_blocks: Sequence[int], pool_blocks: int, kind: str,
                rng: np.random.Generator) -> List[np.ndarray]:
    """Draw disjoint per-request block tables from a pool.

    kind:
      "random"      disjoint slices of one random permutation of the pool
      "fragmented"  as random, then repaired so that no two consecutive
                    logical blocks of a request are physically adjacent
      "contiguous"  each request gets one physically contiguous extent
                    (extents placed in random order, random gaps)
      "runs"        random-length physically contiguous extents of 1..8 blocks,
                    shuffled: exercises coalescing of adjacent blocks
    """
    n_blocks = [int(x) for x in n_blocks]
    total = sum(n_blocks)
    if total > pool_blocks:
        raise ValueError("pool too small for the batch")
    out: List[np.ndarray] = []
    if kind in ("random", "fragmented"):
        perm = rng.permutation(pool_blocks).astype(np.int32)
        pos = 0
        for n in n_blocks:
            t = perm[pos:pos + n].copy()
            pos += n
            if kind == "fragmented":
                _repair_adjacent(t, rng)
            out.append(t)
    elif kind == "contiguous":
        order = rng.permutation(len(n_blocks))
        slack = pool_blocks - total
        cuts = np.sort(rng.integers(0, slack + 1, size=len(n_blocks)))
        gaps = np.diff(np.concatenate([[0], cuts]))
        start = 0
        tabs: List[Optional[np.ndarray]] = [None] * len(n_blocks)
        for k, r in enumerate(order):
            start += int(gaps[k])
            tabs[r] = np.arange(start, start + n_blocks[r], dtype=np.int32)
            start += n_blocks[r]
        out = [t for t in tabs]  # type: ignore[misc]
    elif kind == "runs":
        # cut the pool into extents of 1..8 blocks, shuffle the extents, deal
        # them out; a request's table is then a sequence of short extents.
        lens = []
        left = pool_blocks
        while left > 0:
            k = int(min(left, rng.integers(1, 9)))
            lens.append(k)
            left -= k
        starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
        order = rng.permutation(len(lens))
        stream = np.concatenate(
            [np.arange(starts[e], starts[e] + lens[e]) for e in order]
        ).astype(np.int32)
        pos = 0
        for n in n_blocks:
            out.append(stream[pos:pos + n].copy())
            pos += n
    else:
        raise ValueError(kind)
    return out


def _sides(hit, app, bs, kind, pool_factor, pool_blocks, seed):
    nb = _blocks_needed(hit, app, bs)
    if pool_blocks is None:
        pool_blocks = int(np.ceil(pool_factor * int(nb.sum())))
    rs = np.random.Generator(np.random.PCG64(seed + 100))
    rd = np.random.Generator(np.random.PCG64(seed + 150))
    src = Side(pool_blocks, make_tables(nb, pool_blocks, kind, rs))
    dst = Side(pool_blocks, make_tables(nb, pool_blocks, kind, rd))
    return src, dst


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def config(index: int, n_requests: Optional[int] = None,
           token_scale: float = 1.0) -> Workload:
    """Workload ``index`` (1..5).

    ``n_requests`` and ``token_scale`` shrink the batch (fewer requests,
    shorter prefixes) for cases a CPU has to finish in seconds; with the
    defaults the full-size configuration is returned.  Lengths are drawn first
    and then scaled, so the scaled batch keeps the shape of the full one.
    """
    seed = BASE_SEED + index
    rng = np.random.Generator(np.random.PCG64(seed))

    def scaled(x):
        return np.maximum(1, np.rint(np.asarray(x, dtype=np.float64) * token_scale)).astype(np.uint32)

    if index == 1:
        # tiny MLA-style cache: 576 bf16 per token, 16-token blocks
        lay = Layout(2, 16, (1152,))
        R = n_requests or 4
        hit = scaled(np.full(R, 1000))
        app = np.zeros(R, dtype=np.uint32)
        src, dst = _sides(hit, app, lay.block_tokens, "random", None, 512, seed)
        return Workload("cfg1_tiny_mla", 1, lay, hit, app, src, dst, "bf16_uniform", seed)
    if index == 2:
        # GQA: separate K and V planes of 8 heads x 128 dims bf16
        lay = Layout(32, 64, (2048, 2048))
        R = n_requests or 64
        hit = scaled(rng.integers(16 * 1024, 64 * 1024 + 1, size=R))
        app = rng.integers(256, 1024 + 1, size=R).astype(np.uint32)
        src, dst = _sides(hit, app, lay.block_tokens, "random", 1.1, None, seed)
        return Workload("cfg2_gqa", 2, lay, hit, app, src, dst, "bf16_uniform", seed)
    if index in (3, 5):
        # MLA: 512 latent + 64 rope bf16 per token
        lay = Layout(61, 64, (1152,))
        R = n_requests or 128
        draw_rng = np.random.Generator(np.random.PCG64(BASE_SEED + 3))
        raw = np.minimum(draw_rng.lognormal(np.log(32768.0), 0.5, size=R), 131072.0)
        hit = scaled(raw)
        app = np.maximum(1, np.rint(hit.astype(np.float64) * 5.0 / 95.0)).astype(np.uint32)
        src, dst = _sides(hit, app, lay.block_tokens, "random", 1.1, None, BASE_SEED + 3)
        name = "cfg3_mla" if index == 3 else "cfg5_mla_streamed"
        w = Workload(name, index, lay, hit, app, src, dst, "bf16_uniform", seed)
        if index == 5:
            w.notes.update(compute_us=200, dev_slots=2, host_slots=2)
        return w
    if index == 4:
        # fp8 MLA: 512 e4m3 + 4 fp32 scales + 64 bf16 rope = 656 opaque bytes
        lay = Layout(61, 64, (656,))
        R = n_requests or 256
        hit = scaled(rng.integers(8 * 1024, 128 * 1024 + 1, size=R))
        app = rng.integers(256, 1024 + 1, size=R).astype(np.uint32)
        src, dst = _sides(hit, app, lay.block_tokens, "fragmented", 1.1, None, seed)
        return Workload("cfg4_fp8_mla", 4, lay, hit, app, src, dst, "bytes", seed)
    raise ValueError("config index must be 1..5")


def tiny(seed: int, n_requests: int, block_tokens: int, row_bytes: Sequence[int],
         pool_blocks: int, max_tokens: int, kind: str = "random",
         n_layers: int = 1, allow_zero_hit: bool = True) -> Workload:
    """Small adversarial batch: ragged hits (including 0 and exact block
    multiples), a boundary block shared by hit and appended rows."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lo = 0 if allow_zero_hit else 1
    hit = rng.integers(lo, max_tokens + 1, size=n_requests).astype(np.uint32)
    # force a few special lengths when there is room
    if n_requests >= 3 and max_tokens >= block_tokens:
        hit[0] = block_tokens * max(1, max_tokens // block_tokens // 2)  # exact multiple
        hit[1] = min(max_tokens, int(hit[1]) | 1)                        # odd
    app = rng.integers(0, block_tokens * 2 + 1, size=n_requests).astype(np.uint32)
    lay = Layout(n_layers, block_tokens, tuple(int(x) for x in row_bytes))
    nb = _blocks_needed(hit, app, block_tokens)
    if int(nb.sum()) > pool_blocks:
        # shrink from the back until the batch fits
        for r in range(n_requests - 1, -1, -1):
            hit[r] = 0
            app[r] = 0
            nb = _blocks_needed(hit, app, block_tokens)
            if int(nb.sum()) <= pool_blocks:
                break
    rs = np.random.Generator(np.random.PCG64(seed + 100))
    rd = np.random.Generator(np.random.PCG64(seed + 150))
    src = Side(pool_blocks, make_tables(nb, pool_blocks, kind, rs))
    dst = Side(pool_blocks, make_tables(nb, pool_blocks, kind, rd))
    return Workload(f"tiny_{seed}", 0, lay, hit, app, src, dst, "bytes", seed)


def from_trace(max_len_k: int = 64, n_requests: int = 16, seed: int = 0,
               layout: Optional[Layout] = None, kind: str = "random") -> Workload:
    """A batch of concurrent requests taken from the synthetic agent trace: one turn each of
    ``n_requests`` different trajectories.  The turn's context is the request's hit prefix,
    its appended tokens the tail.  Default layout: the 61-layer MLA cache of config 3."""
    t = agent_trace(max_len_k, seed=seed)
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 600 + seed))
    trajs = rng.choice(t.n_traj, size=n_requests, replace=False)
    rows = []
    for i in trajs:
        idx = np.flatnonzero(t.traj == i)
        rows.append(int(rng.choice(idx[1:] if idx.size > 1 else idx)))      # not the first turn: nothing cached there
    hit = t.context[rows].astype(np.uint32)
    app = t.append[rows].astype(np.uint32)
    lay = layout or Layout(61, 64, (1152,))
    src, dst = _sides(hit, app, lay.block_tokens, kind, 1.1, None, BASE_SEED + 600 + seed)
    return Workload(f"trace{max_len_k}k_{n_requests}req", 0, lay, hit, app, src, dst, "bytes", BASE_SEED + 600 + seed)


# --------------------------------------------------------------------------
# pool fills
# --------------------------------------------------------------------------

def _bf16_uniform(n_elems: int, rng: np.random.Generator) -> np.ndarray:
    """n_elems bf16 bit patterns, values uniform in [-1, 1] (round to nearest even)."""
    f = rng.uniform(-1.0, 1.0, size=n_elems).astype(np.float32)
    u = f.view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return u.astype(np.uint16)


def _fill_rng(w: Workload, layer: int, plane: int, which: str) -> np.random.Generator:
    salt = {"src": 0, "dst": 1, "payload": 2}[which]
    return np.random.Generator(np.random.PCG64([w.seed + 200, layer, plane, salt]))


def fill_pool(w: Workload, layer: int, which: str = "src") -> List[np.ndarray]:
    """Fully random pool contents for one layer: a list of uint8 arrays, one
    per plane, each ``pool_blocks * block_tokens * row_bytes`` long."""
    side = w.src if which == "src" else w.dst
    out = []
    for p, row in enumerate(w.layout.row_bytes):
        n = side.pool_blocks * w.layout.block_tokens * row
        rng = _fill_rng(w, layer, p, which)
        if w.fill == "bf16_uniform" and row % 2 == 0:
            out.append(_bf16_uniform(n // 2, rng).view(np.uint8))
        else:
            out.append(rng.integers(0, 256, size=n, dtype=np.uint8))
    return out


def fill_pool_fast(w: Workload, layer: int, which: str = "src",
                   tile_bytes: int = 1 << 24) -> List[np.ndarray]:
    """Pool contents for full-size runs, cheap to produce for tens of GB.

    A random tile (same distribution as ``fill_pool``) is repeated over the
    pool; then the first 8 bytes of every token row are replaced by a tag
    ``(layer << 56) | (plane << 48) | physical_row`` so that every row of every
    layer and plane is distinct and names where it came from.
    """
    side = w.src if which == "src" else w.dst
    out = []
    for p, row in enumerate(w.layout.row_bytes):
        if row % 8:
            raise ValueError("fast fill needs rows that are a multiple of 8 bytes")
        n_rows = side.pool_blocks * w.layout.block_tokens
        n = n_rows * row
        rng = _fill_rng(w, layer, p, which)
        tb = min(tile_bytes, n)
        tb -= tb % 8
        if w.fill == "bf16_uniform":
            tile = _bf16_uniform(tb // 2, rng).view(np.uint8)
        else:
            tile = rng.integers(0, 256, size=tb, dtype=np.uint8)
        buf = np.empty(n, dtype=np.uint8)
        pos = 0
        while pos < n:
            k = min(tb, n - pos)
            buf[pos:pos + k] = tile[:k]
            pos += k
        tags = (np.uint64(layer & 0xFF) << np.uint64(56)) | (np.uint64(p) << np.uint64(48)) \
            | np.arange(n_rows, dtype=np.uint64)
        buf.view(np.uint64).reshape(n_rows, row // 8)[:, 0] = tags
        out.append(buf)
    return out


def sentinel_pool(w: Workload, which: str = "dst", byte: int = 0xA5) -> List[np.ndarray]:
    """A pool filled with one byte value, to show which bytes a scatter wrote."""
    side = w.src if which == "src" else w.dst
    return [np.full(side.pool_blocks * w.layout.block_tokens * row, byte, dtype=np.uint8)
            for row in w.layout.row_bytes]


def random_payload(w: Workload, layer: int, n_bytes: int) -> np.ndarray:
    """An arbitrary byte string of a given length (a transfer buffer's content)."""
    rng = _fill_rng(w, layer, 0, "payload")
    return rng.integers(0, 256, size=n_bytes, dtype=np.uint8)


from .agent_trace import PUBLISHED as PUBLISHED_TRACE_STATS  # noqa: E402  (needs BASE_SEED above)
from .agent_trace import AgentTrace, agent_trace  # noqa: E402
