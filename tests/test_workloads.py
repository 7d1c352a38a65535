"""The seeded input generators: shapes, determinism and table structure."""
import numpy as np
import pytest

import kvl_workloads as W


@pytest.mark.parametrize("idx", [1, 2, 3, 4, 5])
def test_config_shapes_and_tables(idx):
    w = W.config(idx)
    w2 = W.config(idx)
    bs = w.layout.block_tokens
    assert np.array_equal(w.hit, w2.hit) and np.array_equal(w.app, w2.app)
    for side, side2 in ((w.src, w2.src), (w.dst, w2.dst)):
        used = np.concatenate(side.tables)
        assert used.min() >= 0 and used.max() < side.pool_blocks
        assert np.unique(used).size == used.size            # disjoint, no repeats
        for r, t in enumerate(side.tables):
            assert t.dtype == np.int32
            assert t.size == -(-(int(w.hit[r]) + int(w.app[r])) // bs)
            assert np.array_equal(t, side2.tables[r])        # seeded
    assert not all(np.array_equal(a, b) for a, b in zip(w.src.tables, w.dst.tables))


def test_config_statistics():
    w1 = W.config(1)
    assert w1.n_requests == 4 and np.all(w1.hit == 1000) and w1.src.pool_blocks == 512
    assert w1.layout == W.Layout(2, 16, (1152,))
    w2 = W.config(2)
    assert w2.layout == W.Layout(32, 64, (2048, 2048)) and w2.n_requests == 64
    assert w2.hit.min() >= 16384 and w2.hit.max() <= 65536
    assert w2.app.min() >= 256 and w2.app.max() <= 1024
    nb = sum(t.size for t in w2.src.tables)
    assert w2.src.pool_blocks == int(np.ceil(1.1 * nb))
    w3 = W.config(3)
    assert w3.layout == W.Layout(61, 64, (1152,)) and w3.n_requests == 128
    assert w3.hit.max() <= 131072
    assert 24000 < np.median(w3.hit) < 42000                # lognormal, median 32K
    rate = w3.hit.sum() / (w3.hit.sum() + w3.app.sum())
    assert abs(rate - 0.95) < 1e-3
    w4 = W.config(4)
    assert w4.layout == W.Layout(61, 64, (656,)) and w4.n_requests == 256
    assert w4.hit.min() >= 8192 and w4.hit.max() <= 131072
    for side in (w4.src, w4.dst):                            # fully fragmented
        for t in side.tables:
            assert not np.any(np.abs(np.diff(t.astype(np.int64))) == 1)
    w5 = W.config(5)
    assert np.array_equal(w5.hit, w3.hit) and w5.notes["compute_us"] == 200


def test_trace_statistics_are_consistent():
    # Table 2's 64K set: mean context 32721, mean append 429 -> the 98.7 % hit
    # rate quoted in Section 3 for the same traces
    assert round(100 * 32721 / (32721 + 429), 1) == 98.7


def test_scaled_config_keeps_shape():
    w = W.config(2, n_requests=6, token_scale=1 / 64)
    assert w.n_requests == 6 and w.layout.row_bytes == (2048, 2048)
    assert w.hit.min() >= 256 and w.hit.max() <= 1024
    assert any(int(h) % w.layout.block_tokens for h in w.hit)     # ragged tails survive


def test_table_kinds():
    rng = np.random.Generator(np.random.PCG64(3))
    for kind in ("random", "fragmented", "contiguous", "runs"):
        tabs = W.make_tables([5, 9, 1, 0, 14], 40, kind, rng)
        used = np.concatenate(tabs)
        assert np.unique(used).size == used.size == 29 and used.max() < 40
    c = W.make_tables([6, 4], 32, "contiguous", rng)
    assert all(np.all(np.diff(t) == 1) for t in c)
    r = W.make_tables([200], 256, "runs", rng)[0]
    assert np.any(np.diff(r) == 1) and np.any(np.diff(r) != 1)


def test_fills():
    w = W.config(1)
    a = W.fill_pool(w, 0)[0]
    b = W.fill_pool(w, 0)[0]
    c = W.fill_pool(w, 1)[0]
    assert a.tobytes() == b.tobytes() and a.tobytes() != c.tobytes()
    assert a.size == 512 * 16 * 1152
    # bf16 patterns decode to values in [-1, 1]
    f = (a.view(np.uint16).astype(np.uint32) << 16).view(np.float32)
    assert f.min() >= -1.0 and f.max() <= 1.0 and abs(float(f.mean())) < 0.01
    fast = W.fill_pool_fast(w, 1, tile_bytes=1 << 16)[0]
    tags = fast.view(np.uint64).reshape(-1, 1152 // 8)[:, 0]
    assert np.array_equal(tags & np.uint64(0xFFFFFFFFFFFF), np.arange(512 * 16, dtype=np.uint64))
    assert np.all(tags >> np.uint64(56) == 1)


# --------------------------------------------------------------------------
# agent trajectories shaped like the paper's trace datasets (Section 7.1, table of
# agent trace statistics)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("max_len_k", [32, 48, 64])
def test_agent_trace_reproduces_the_published_averages(max_len_k):
    pub = W.PUBLISHED_TRACE_STATS[max_len_k]
    big = W.agent_trace(max_len_k, n_traj=4000).stats()          # little sampling noise: within 5 %
    for k, v in pub.items():
        assert big[k] == pytest.approx(v, rel=0.05), (k, big[k], v)
    t = W.agent_trace(max_len_k)                                 # the datasets' own size: 500 trajectories
    s = t.stats()
    for k, v in pub.items():
        assert s[k] == pytest.approx(v, rel=0.10), (k, s[k], v)
    assert t.n_traj == 500 and int(t.traj.max()) == 499
    # every request stays within MaxLen, and the cached prefix dominates it (Section 3: hit rates of 95 % and more)
    assert int((t.context + t.append + t.gen).max()) <= max_len_k * 1024
    assert s["hit_rate"] > 0.95
    # a trajectory's context at a turn is everything before it
    a = np.flatnonzero(t.traj == 7)
    assert np.array_equal(t.context[a][1:], t.context[a][0] + np.cumsum(t.append[a] + t.gen[a])[:-1])
    # seeded
    u = W.agent_trace(max_len_k)
    assert np.array_equal(t.context, u.context) and np.array_equal(t.append, u.append)
    assert not np.array_equal(W.agent_trace(max_len_k, seed=1).context[:100], t.context[:100])


def test_batch_drawn_from_the_trace_is_a_valid_workload():
    w = W.from_trace(64, 16)
    assert w.n_requests == 16 and w.layout.block_tokens == 64 and w.layout.row_bytes == (1152,)
    for side in (w.src, w.dst):
        ids = np.concatenate(side.tables)
        assert ids.min() >= 0 and ids.max() < side.pool_blocks and np.unique(ids).size == ids.size
        for r, t in enumerate(side.tables):
            assert t.size == -(-(int(w.hit[r]) + int(w.app[r])) // 64)
    assert np.all(w.hit > 0) and np.all(w.hit.astype(np.int64) + w.app <= 64 * 1024)
    assert float(w.hit.sum()) / float(w.hit.sum() + w.app.sum()) > 0.95
    v = W.from_trace(64, 16)
    assert np.array_equal(v.hit, w.hit) and all(np.array_equal(a, b) for a, b in zip(v.src.tables, w.src.tables))
