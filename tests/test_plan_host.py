"""Host logic of the library (no GPU): kvl_plan's descriptors, checked against the oracle.

A KVL_HOST_ONLY plan yields the copy descriptors without touching a device.
Replaying them with NumPy slices (a row-span copy per descriptor, which is all
a descriptor means) must reproduce the oracle's pack and unpack bit for bit.
"""
import numpy as np
import pytest

import kvl_workloads as W
import oracle
import paper_2602_21548_amd as K


def host_plan(w, side, flags, **tuning):
    s = w.src if side == "src" else w.dst
    lay = K.make_layout(w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes, s.pool_blocks)
    return K.kvl_plan(lay, w.hit, w.app, s.tables, flags | K.KVL_HOST_ONLY, **tuning)


def replay_pack(plan, row_bytes, pools):
    T = plan.hit_tokens
    out = np.zeros(plan.payload_bytes, dtype=np.uint8)
    base = 0
    for p, row in enumerate(row_bytes):
        for pool_row, xfer_row, n, _ in plan.units():
            a, b, k = int(pool_row) * row, base + int(xfer_row) * row, int(n) * row
            out[b:b + k] = pools[p][a:a + k]
        base += T * row
    return out


def replay_unpack(plan, row_bytes, xfer, pools):
    T = plan.hit_tokens
    base = 0
    for p, row in enumerate(row_bytes):
        for pool_row, xfer_row, n, _ in plan.units():
            a, b, k = int(pool_row) * row, base + int(xfer_row) * row, int(n) * row
            pools[p][a:a + k] = xfer[b:b + k]
        base += T * row


CASES = [
    ("tiny-random", lambda: W.tiny(101, 6, 16, (48,), 64, 90)),
    ("tiny-runs-2planes", lambda: W.tiny(102, 7, 4, (32, 16), 200, 60, kind="runs")),
    ("tiny-contig", lambda: W.tiny(103, 5, 8, (16,), 100, 120, kind="contiguous")),
    ("tiny-oddrow", lambda: W.tiny(104, 4, 3, (5,), 60, 40)),
    ("cfg1", lambda: W.config(1)),
    ("cfg2-small", lambda: W.config(2, n_requests=5, token_scale=1 / 128)),
    ("cfg3-small", lambda: W.config(3, n_requests=8, token_scale=1 / 64)),
    ("cfg4-small", lambda: W.config(4, n_requests=8, token_scale=1 / 128)),
]


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("unit_bytes", [0, 4096, 1 << 20])
def test_descriptors_reproduce_the_oracle(name, make, unit_bytes):
    w = make()
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    g = host_plan(w, "src", K.KVL_GATHER, unit_bytes=unit_bytes)
    assert g.payload_bytes == oracle.payload_bytes(w.hit, rows)
    assert g.hit_tokens == oracle.total_hit_tokens(w.hit)
    src = W.fill_pool(w, 0, "src")
    want = oracle.pack(bs, rows, w.hit, w.src.tables, src)
    assert replay_pack(g, rows, src).tobytes() == want.tobytes()

    s = host_plan(w, "dst", K.KVL_SCATTER, unit_bytes=unit_bytes)
    got = W.sentinel_pool(w, "dst")
    ref = W.sentinel_pool(w, "dst")
    replay_unpack(s, rows, want, got)
    oracle.unpack(bs, rows, w.hit, w.dst.tables, want, ref)
    for a, b in zip(got, ref):
        assert a.tobytes() == b.tobytes()


def test_descriptors_tile_the_transfer_buffer():
    w = W.tiny(105, 9, 16, (64,), 300, 200, kind="runs")
    for ub in (0, 256, 2048, 1 << 16):
        p = host_plan(w, "src", K.KVL_GATHER, unit_bytes=ub)
        u = p.units().astype(np.int64)
        assert np.all(u[:, 2] > 0)
        assert u[0, 1] == 0
        assert np.array_equal(u[1:, 1], u[:-1, 1] + u[:-1, 2])       # dense, in order
        assert u[-1, 1] + u[-1, 2] == p.hit_tokens
        max_rows = max(1, (ub or (128 << 10)) // 64)
        assert u[:, 2].max() <= max_rows
        assert np.all(u[:, 0] + u[:, 2] <= w.src.pool_blocks * 16)


def test_merging_of_adjacent_blocks():
    bs, row = 16, 32
    lay = K.make_layout(1, bs, (row,), 64)
    tbl = [np.arange(10, 30, dtype=np.int32)]                  # 20 physically consecutive blocks
    hit, app = [20 * bs - 3], [0]
    merged = K.kvl_plan(lay, hit, app, tbl, K.KVL_GATHER | K.KVL_HOST_ONLY, unit_bytes=1 << 20)
    assert merged.n_units == 1 and merged.units()[0].tolist()[:3] == [10 * bs, 0, 20 * bs - 3]
    split = K.kvl_plan(lay, hit, app, tbl, K.KVL_GATHER | K.KVL_HOST_ONLY, unit_bytes=bs * row * 4)
    n = split.units()[:, 2]
    assert split.n_units == 5 and n.max() - n.min() <= 1      # even split
    single = K.kvl_plan(lay, hit, app, tbl, K.KVL_GATHER | K.KVL_HOST_ONLY | K.KVL_NO_MERGE, unit_bytes=1 << 20)
    assert single.n_units == 20
    # a descending table has no run to merge
    rev = K.kvl_plan(lay, hit, app, [tbl[0][::-1].copy()], K.KVL_GATHER | K.KVL_HOST_ONLY, unit_bytes=1 << 20)
    assert rev.n_units == 20
    # fully fragmented tables: one descriptor per block
    w = W.config(4, n_requests=6, token_scale=1 / 64)
    p = host_plan(w, "src", K.KVL_GATHER, unit_bytes=64 * 656)
    assert p.n_units == sum(-(-int(h) // 64) for h in w.hit)


ERR = {oracle.OK: K.KVL_OK, oracle.E_TABLE: K.KVL_ERANGE, oracle.E_BLOCK: K.KVL_ERANGE, oracle.E_DUP: K.KVL_EALIAS}


@pytest.mark.parametrize("case", [
    dict(hit=[9, 2], app=[1, 2], tables=[[1, 2, 3], [5]]),
    dict(hit=[9, 2], app=[4, 2], tables=[[1, 2, 3], [5]]),            # table too short
    dict(hit=[9, 2], app=[1, 2], tables=[[1, 2, 10], [5]]),           # id == pool_blocks
    dict(hit=[9, 2], app=[1, 2], tables=[[1, -1, 3], [5]]),           # negative id
    dict(hit=[9, 2], app=[1, 2], tables=[[1, 2, 3], [2]]),            # duplicate destination
    dict(hit=[8, 2], app=[4, 6], tables=[[1, 2, 3], [5, 3]]),         # shared block holds appended rows only
    dict(hit=[0, 0], app=[0, 3], tables=[[], [7]]),
])
def test_validation_agrees_with_the_oracle(case):
    bs, pool = 4, 10
    lay = K.make_layout(1, bs, (16,), pool)
    tabs = [np.array(t, dtype=np.int32) for t in case["tables"]]
    for scatter in (False, True):
        want = ERR[oracle.check(bs, pool, case["hit"], case["app"], tabs, scatter)]
        flags = (K.KVL_SCATTER if scatter else K.KVL_GATHER) | K.KVL_HOST_ONLY
        try:
            K.kvl_plan(lay, case["hit"], case["app"], tabs, flags)
            got = K.KVL_OK
        except K.KvlError as e:
            got = e.code
        assert got == want, (case, scatter)


def test_argument_errors():
    tabs = [np.array([0], np.int32)]
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(K.make_layout(1, 0, (16,), 4), [1], [0], tabs, K.KVL_GATHER | K.KVL_HOST_ONLY)
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(K.make_layout(1, 4, (0,), 4), [1], [0], tabs, K.KVL_GATHER | K.KVL_HOST_ONLY)
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(K.make_layout(1, 4, (16,), 4), [1], [0], tabs, K.KVL_HOST_ONLY)      # neither gather nor scatter
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(K.make_layout(1, 4, (16,), 4), [1], [0], tabs, K.KVL_GATHER | K.KVL_HOST_ONLY, block_threads=96)
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(K.KvlError) as e:                                               # 2^32 pool rows
        K.kvl_plan(K.make_layout(1, 64, (16,), 1 << 26), [1], [0], tabs, K.KVL_GATHER | K.KVL_HOST_ONLY)
    assert e.value.code == K.KVL_ERANGE
    # a host-only plan cannot be executed (checked before any pointer is used)
    p = K.kvl_plan(K.make_layout(1, 4, (16,), 4), [1], [0], tabs, K.KVL_GATHER | K.KVL_HOST_ONLY)
    from paper_2602_21548_amd import binding as B
    import ctypes as C
    arr = (C.c_void_p * 1)(0x1000)
    assert B._lib.kvl_pack_layer(p.handle, arr, 0x1000, 1 << 20, None) == K.KVL_EINVAL
    assert B._lib.kvl_unpack_layer(p.handle, 0x1000, 1 << 20, arr, None) == K.KVL_EINVAL


def test_empty_batch_plan():
    lay = K.make_layout(1, 16, (32,), 8)
    p = K.kvl_plan(lay, [], [], [], K.KVL_GATHER | K.KVL_HOST_ONLY)
    assert p.payload_bytes == 0 and p.n_units == 0 and p.chunks(1024) == []


def test_h2d_chunks_cover_the_payload():
    w = W.config(2, n_requests=5, token_scale=1 / 128)
    p = host_plan(w, "dst", K.KVL_SCATTER, unit_bytes=16384)
    T, rows = p.hit_tokens, w.layout.row_bytes
    for cb in (16384, 100000, 1 << 20, 1 << 30):
        ch = p.chunks(cb)
        pos, base = 0, 0
        for plane, row in enumerate(rows):
            mine = [c for c in ch if c["plane"] == plane]
            assert mine[0]["unit_begin"] == 0 and mine[-1]["unit_end"] == p.n_units
            for a, b in zip(mine, mine[1:]):
                assert a["unit_end"] == b["unit_begin"]
            for c in mine:
                assert 0 < c["bytes"] <= cb and c["host_offset"] == pos
                pos += c["bytes"]
            base += T * row
            assert pos == base
        assert pos == p.payload_bytes
    with pytest.raises(K.KvlError) as e:
        p.chunks(1024)                      # smaller than one descriptor
    assert e.value.code == K.KVL_ESPACE


# --------------------------------------------------------------------------
# token ranges: the appended tail and the whole prompt
# --------------------------------------------------------------------------

def _range_of(w, flag):
    zero = np.zeros_like(w.hit)
    if flag == K.KVL_TOKENS_APPEND:
        return w.hit, w.app
    if flag == K.KVL_TOKENS_ALL:
        return zero, w.hit + w.app
    return zero, w.hit


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("flag", [K.KVL_TOKENS_APPEND, K.KVL_TOKENS_ALL], ids=["append", "all"])
def test_range_descriptors_reproduce_the_oracle(name, make, flag):
    w = make()
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    first, count = _range_of(w, flag)
    for ub in (0, 2048):
        g = host_plan(w, "src", K.KVL_GATHER | flag, unit_bytes=ub)
        assert g.hit_tokens == int(count.astype(np.int64).sum())
        assert g.payload_bytes == oracle.payload_bytes(count, rows)
        src = W.fill_pool(w, 0, "src")
        want = oracle.pack_range(bs, rows, first, count, w.src.tables, src)
        assert replay_pack(g, rows, src).tobytes() == want.tobytes()
        s = host_plan(w, "dst", K.KVL_SCATTER | flag, unit_bytes=ub)
        got, ref = W.sentinel_pool(w, "dst"), W.sentinel_pool(w, "dst")
        replay_unpack(s, rows, want, got)
        oracle.unpack_range(bs, rows, first, count, w.dst.tables, want, ref)
        for a, b in zip(got, ref):
            assert a.tobytes() == b.tobytes()


def test_range_merging_and_flags():
    bs, row = 16, 32
    lay = K.make_layout(1, bs, (row,), 64)
    tbl = [np.arange(10, 30, dtype=np.int32)]
    # tail starts mid-block and runs over 3 physically consecutive blocks: one run
    p = K.kvl_plan(lay, [5 * bs + 3], [2 * bs + 4], tbl, K.KVL_GATHER | K.KVL_HOST_ONLY | K.KVL_TOKENS_APPEND,
                   unit_bytes=1 << 20)
    assert p.units()[:, :3].tolist() == [[15 * bs + 3, 0, 2 * bs + 4]]
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(lay, [5], [4], tbl, K.KVL_GATHER | K.KVL_HOST_ONLY | K.KVL_TOKENS_APPEND | K.KVL_TOKENS_ALL)
    assert e.value.code == K.KVL_EINVAL


@pytest.mark.parametrize("case", [
    dict(hit=[0, 0], app=[5, 3], tables=[[1, 2], [2, 3]]),     # both tails touch block 2
    dict(hit=[0, 0], app=[4, 3], tables=[[1, 2], [2, 3]]),
    dict(hit=[0, 4], app=[5, 3], tables=[[1, 2], [2, 3]]),     # second tail starts in block 3
    dict(hit=[3, 4], app=[0, 0], tables=[[1], [1]]),           # hit blocks alias, tails are empty
])
def test_range_validation_agrees_with_the_oracle(case):
    bs, pool = 4, 8
    lay = K.make_layout(1, bs, (16,), pool)
    tabs = [np.array(t, dtype=np.int32) for t in case["tables"]]
    hit, app = np.array(case["hit"], np.uint32), np.array(case["app"], np.uint32)
    want = ERR[oracle.check_range_scatter(bs, pool, hit, app, tabs)]
    try:
        K.kvl_plan(lay, hit, app, tabs, K.KVL_SCATTER | K.KVL_HOST_ONLY | K.KVL_TOKENS_APPEND)
        got = K.KVL_OK
    except K.KvlError as e:
        got = e.code
    assert got == want, case


# --------------------------------------------------------------------------
# storage layout: descriptors carry the Full-Block index
# --------------------------------------------------------------------------

def replay_to_fullblocks(plan, lay, layer, pools, buf):
    """What a descriptor means for the storage layout, spelt out with NumPy slices."""
    bs, rows, L = lay.block_tokens, lay.row_bytes, lay.n_layers
    fb, nfb = plan.fullblock_geometry()
    lb = fb // L
    po = 0
    for p, row in enumerate(rows):
        for pool_row, _, n, bi in plan.units():
            w = int(pool_row) % bs
            dst = int(bi) * fb + layer * lb + po + w * row
            src = int(pool_row) * row
            buf[dst:dst + int(n) * row] = pools[p][src:src + int(n) * row]
        po += bs * row


@pytest.mark.parametrize("name,make", CASES[:4] + CASES[5:6], ids=[c[0] for c in CASES[:4] + CASES[5:6]])
@pytest.mark.parametrize("flag", [0, K.KVL_TOKENS_APPEND, K.KVL_TOKENS_ALL], ids=["hit", "append", "all"])
def test_fullblock_descriptors_reproduce_the_oracle(name, make, flag):
    w = make()
    L = 3
    lay = W.Layout(L, w.layout.block_tokens, w.layout.row_bytes)
    bs, rows = lay.block_tokens, lay.row_bytes
    first, count = _range_of(w, flag)
    klay = K.make_layout(L, bs, rows, w.src.pool_blocks)
    plan = K.kvl_plan(klay, w.hit, w.app, w.src.tables, K.KVL_GATHER | K.KVL_HOST_ONLY | K.KVL_NO_MERGE | flag,
                      unit_bytes=4096)
    fb, nfb = plan.fullblock_geometry()
    assert fb == oracle.fullblock_bytes(bs, L, rows) and nfb == oracle.fullblock_count(bs, first, count)
    got = np.full(nfb * fb, 0x5A, dtype=np.uint8)
    want = np.full(nfb * fb, 0x5A, dtype=np.uint8)
    for l in range(L):
        pools = W.fill_pool(w, l, "src")
        replay_to_fullblocks(plan, lay, l, pools, got)
        oracle.pool_to_fullblocks(bs, L, rows, first, count, w.src.tables, l, pools, want)
    assert got.tobytes() == want.tobytes()
    # descriptors of an unmerged plan never span blocks
    u = plan.units().astype(np.int64)
    assert np.all(u[:, 0] % bs + u[:, 2] <= bs)


@pytest.mark.parametrize("seed", range(24))
def test_random_batches_all_ranges(seed):
    """Random small batches (all table kinds, ragged hits, 1-3 planes, odd rows): descriptors
    replayed on the host equal the oracle for the hit prefix, the tail and the whole prompt."""
    rng = np.random.Generator(np.random.PCG64(9000 + seed))
    bs = int(rng.choice([1, 2, 3, 8, 16, 64]))
    planes = int(rng.integers(1, 4))
    rows = tuple(int(rng.choice([5, 16, 36, 48, 656, 1152])) for _ in range(planes))
    kind = ["random", "fragmented", "contiguous", "runs"][seed % 4]
    R = int(rng.integers(1, 9))
    max_tokens = int(rng.integers(1, 6 * bs + 2))
    pool_blocks = R * (max_tokens // bs + 4) + 3
    w = W.tiny(9000 + seed, R, bs, rows, pool_blocks, max_tokens, kind=kind)
    ub = int(rng.choice([0, 64, 700, 5000]))
    for flag in (0, K.KVL_TOKENS_APPEND, K.KVL_TOKENS_ALL):
        first, count = _range_of(w, flag)
        g = host_plan(w, "src", K.KVL_GATHER | flag, unit_bytes=ub)
        src = W.fill_pool(w, 0, "src")
        want = oracle.pack_range(bs, rows, first, count, w.src.tables, src)
        assert replay_pack(g, rows, src).tobytes() == want.tobytes()
        s = host_plan(w, "dst", K.KVL_SCATTER | flag, unit_bytes=ub)
        got, ref = W.sentinel_pool(w, "dst"), W.sentinel_pool(w, "dst")
        replay_unpack(s, rows, want, got)
        oracle.unpack_range(bs, rows, first, count, w.dst.tables, want, ref)
        for a, b in zip(got, ref):
            assert a.tobytes() == b.tobytes()


def test_hip_errors_are_surfaced_not_swallowed():
    """Without a GPU a device plan must fail with KVL_EHIP and carry the HIP error text."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    lay = K.make_layout(1, 4, (16,), 4)
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(lay, [1], [0], [np.array([0], np.int32)], K.KVL_GATHER)
    assert e.value.code == K.KVL_EHIP and "hip" in str(e.value).lower()


def test_row_index_limits():
    """Descriptors index rows with 32 bits: more than 2^32-1 moved tokens is refused, not wrapped."""
    bs = 1 << 20
    lay = K.make_layout(1, bs, (16,), 4095)                      # 4095 x 2^20 pool rows: just below 2^32
    tbl = np.arange(3072, dtype=np.int32)
    hit = [3 << 30, 3 << 30]                                     # 6 Gi tokens in all
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(lay, hit, [0, 0], [tbl, tbl], K.KVL_GATHER | K.KVL_HOST_ONLY)
    assert e.value.code == K.KVL_ERANGE
    p = K.kvl_plan(lay, hit[:1], [0], [tbl], K.KVL_GATHER | K.KVL_HOST_ONLY, unit_bytes=1 << 30)
    assert p.hit_tokens == 3 << 30 and p.payload_bytes == (3 << 30) * 16
    u = p.units().astype(np.int64)
    assert u[:, 2].sum() == 3 << 30 and (u[:, 2] * 16).max() <= 1 << 30      # descriptors stay within 1 GiB


# --------------------------------------------------------------------------
# paired plans: pool-to-pool descriptors
# --------------------------------------------------------------------------

@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("flag", [0, K.KVL_TOKENS_ALL], ids=["hit", "all"])
def test_paired_descriptors_equal_pack_then_unpack(name, make, flag):
    w = make()
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    first, count = _range_of(w, flag)
    g = host_plan(w, "src", K.KVL_GATHER | flag, unit_bytes=4096)
    s = host_plan(w, "dst", K.KVL_SCATTER | flag)
    m = K.kvl_plan_pair(g, s)
    assert m.hit_tokens == g.hit_tokens and m.payload_bytes == g.payload_bytes
    src = W.fill_pool(w, 0, "src")
    want = W.sentinel_pool(w, "dst")
    oracle.unpack_range(bs, rows, first, count, w.dst.tables,
                        oracle.pack_range(bs, rows, first, count, w.src.tables, src), want)
    got = W.sentinel_pool(w, "dst")
    for p, row in enumerate(rows):
        for src_row, dst_row, n, _ in m.units():
            got[p][int(dst_row) * row:(int(dst_row) + int(n)) * row] = src[p][int(src_row) * row:(int(src_row) + int(n)) * row]
    for a, b in zip(got, want):
        assert a.tobytes() == b.tobytes()
    u = m.units().astype(np.int64)
    assert u[:, 2].sum() == g.hit_tokens


def test_pairing_refuses_mismatched_plans():
    w = W.tiny(120, 4, 16, (48,), 64, 90)
    g = host_plan(w, "src", K.KVL_GATHER)
    s = host_plan(w, "dst", K.KVL_SCATTER)
    for a, b in ((s, s), (g, g)):                                      # wrong kinds
        with pytest.raises(K.KvlError) as e:
            K.kvl_plan_pair(a, b)
        assert e.value.code == K.KVL_EINVAL
    tail = host_plan(w, "dst", K.KVL_SCATTER | K.KVL_TOKENS_ALL)       # other token range
    with pytest.raises(K.KvlError):
        K.kvl_plan_pair(g, tail)
    lay = K.make_layout(1, 16, (64,), w.dst.pool_blocks)               # other row size
    other = K.kvl_plan(lay, w.hit, w.app, w.dst.tables, K.KVL_SCATTER | K.KVL_HOST_ONLY)
    with pytest.raises(K.KvlError):
        K.kvl_plan_pair(g, other)
    m = K.kvl_plan_pair(g, s)
    with pytest.raises(K.KvlError):
        K.kvl_plan_pair(m, s)                                          # a paired plan is not a gather plan


def test_piece_size_follows_the_batch_not_the_rare_adjacent_pair():
    """Descriptors of one launch get the same number of tiles (that of the largest), so a few
    merged runs among single blocks must not set the size: the plan then keeps one descriptor per
    block; a batch whose blocks are all contiguous is still merged into large pieces; and blocks
    a little larger than unit_bytes are halved evenly, merged or not."""
    bs, row = 64, 1024                                     # 64 KiB blocks, two fit the 128 KiB default
    rng = np.random.Generator(np.random.PCG64(77))
    R, per = 8, 40
    perm = rng.permutation(4096)[:R * per].astype(np.int32)
    tables = [np.sort(perm[r * per:(r + 1) * per])[::-1].copy() for r in range(R)]    # descending: never adjacent upwards
    tables[3][10], tables[3][11] = 5000, 5001             # one adjacent pair
    hit = np.full(R, per * bs, dtype=np.uint32)
    app = np.zeros(R, dtype=np.uint32)
    lay = K.make_layout(1, bs, (row,), 8192)
    p = K.kvl_plan(lay, hit, app, tables, K.KVL_GATHER | K.KVL_HOST_ONLY)
    u = p.units()
    assert u[:, 2].max() == bs and p.n_units == R * per, "the merged pair must be split back into blocks"
    # all contiguous: pieces of 128 rows (128 KiB), not of 64
    cont = [np.arange(r * per, (r + 1) * per, dtype=np.int32) for r in range(R)]
    p = K.kvl_plan(lay, hit, app, cont, K.KVL_GATHER | K.KVL_HOST_ONLY)
    assert p.units()[:, 2].max() == 128 and p.n_units == R * per // 2
    # 129 KiB blocks against the 128 KiB limit: halves of 32 rows everywhere, also in the merged pair
    lay2 = K.make_layout(1, bs, (2064,), 8192)
    p = K.kvl_plan(lay2, hit, app, tables, K.KVL_GATHER | K.KVL_HOST_ONLY)
    u = p.units()
    assert set(np.unique(u[:, 2]).tolist()) == {32} and p.n_units == 2 * R * per
