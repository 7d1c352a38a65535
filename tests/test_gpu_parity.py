"""GPU parity: the HIP path against the CPU oracle, bit for bit, through the C ABI.

Every payload is an opaque byte copy, so the bar is exact equality of every
byte (compared as bytes, never as floats: NaN patterns must survive).
"""
import numpy as np
import pytest
import torch

import kvl_workloads as W
import oracle
import paper_2602_21548_amd as K
from gpu_util import dev_plan, pinned_from, planes_to_dev, same_bytes, to_dev, to_host

pytestmark = pytest.mark.gpu

GUARD = 4096

CASES = [
    ("tiny-random", lambda: W.tiny(201, 6, 16, (48,), 64, 90)),
    ("tiny-runs-2planes", lambda: W.tiny(202, 7, 4, (32, 16), 200, 60, kind="runs")),
    ("tiny-contig", lambda: W.tiny(203, 5, 8, (16,), 100, 120, kind="contiguous")),
    ("tiny-oddrow", lambda: W.tiny(204, 4, 3, (5,), 60, 40)),              # byte fallback kernel
    ("tiny-row-mult-of-4", lambda: W.tiny(205, 4, 8, (36,), 60, 100)),     # byte fallback kernel
    ("tiny-3planes", lambda: W.tiny(206, 5, 16, (16, 656, 64), 40, 150)),
    ("tiny-4planes-single-tokens", lambda: W.tiny(214, 8, 1, (16, 32, 48, 2048), 64, 5)),   # KVL_MAX_PLANES, bs = 1
    ("cfg1", lambda: W.config(1)),
    ("cfg2-small", lambda: W.config(2, n_requests=7, token_scale=1 / 32)),
    ("cfg3-small", lambda: W.config(3, n_requests=12, token_scale=1 / 16)),
    ("cfg4-small", lambda: W.config(4, n_requests=12, token_scale=1 / 32)),
    ("trace32k-6req", lambda: W.from_trace(32, 6)),                          # a batch of the synthetic agent trace
    ("token-granular", lambda: W.tiny(215, 9, 1, (1152,), 3000, 300)),       # bs = 1: every token its own block (flat kernel)
    ("token-granular-2planes", lambda: W.tiny(216, 7, 2, (256, 64), 2000, 250, kind="fragmented")),
]


def run_hop(w, layer=0, **tuning):
    """pack on the source pool, unpack into a sentinel pool; compare both with the oracle."""
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool(w, layer, "src")
    want_x = oracle.pack(bs, rows, w.hit, w.src.tables, src, threads=8)
    want_dst = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, want_x, want_dst, threads=8)

    g = dev_plan(w, "src", K.KVL_GATHER, **tuning)
    s = dev_plan(w, "dst", K.KVL_SCATTER, **tuning)
    n = g.payload_bytes
    assert n == want_x.size == s.payload_bytes
    d_src = planes_to_dev(src)
    d_x = torch.full((n + GUARD,), 0x3C, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, d_src, d_x)
    d_dst = planes_to_dev(W.sentinel_pool(w, "dst"))
    K.kvl_unpack_layer(s, d_x, d_dst)
    torch.cuda.synchronize()
    got_x = to_host(d_x)
    assert same_bytes(got_x[:n], want_x), "pack differs from the oracle"
    assert np.all(got_x[n:] == 0x3C), "pack wrote past the payload"
    for p, (a, b) in enumerate(zip(d_dst, want_dst)):
        assert same_bytes(to_host(a), b), f"unpack differs from the oracle in plane {p}"
    for a, b in zip(d_src, src):
        assert same_bytes(to_host(a), b), "pack modified its source"
    g.destroy()
    s.destroy()


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_pack_unpack_default(name, make):
    run_hop(make())


def run_range_hop(w, flag, layer=0, **tuning):
    """The step after a layer's compute: gather a token range from the prefill-side pool,
    merge it into the decode-side pool that already holds other rows."""
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    zero = np.zeros_like(w.hit)
    first, count = (w.hit, w.app) if flag == K.KVL_TOKENS_APPEND else (zero, w.hit + w.app)
    pe = W.fill_pool(w, layer, "dst")               # prefill engine's pool (source of this hop)
    de = W.fill_pool(w, layer, "src")               # decode engine's pool: must keep every other row
    want_x = oracle.pack_range(bs, rows, first, count, w.dst.tables, pe, threads=8)
    want_de = [p.copy() for p in de]
    oracle.unpack_range(bs, rows, first, count, w.src.tables, want_x, want_de, threads=8)
    s_lay = K.make_layout(w.layout.n_layers, bs, rows, w.dst.pool_blocks)
    d_lay = K.make_layout(w.layout.n_layers, bs, rows, w.src.pool_blocks)
    g = K.kvl_plan(s_lay, w.hit, w.app, w.dst.tables, K.KVL_GATHER | flag, **tuning)
    s = K.kvl_plan(d_lay, w.hit, w.app, w.src.tables, K.KVL_SCATTER | flag, **tuning)
    n = g.payload_bytes
    assert n == want_x.size == s.payload_bytes
    d_pe, d_de = planes_to_dev(pe), planes_to_dev(de)
    d_x = torch.full((n + GUARD,), 0x3C, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, d_pe, d_x)
    K.kvl_unpack_layer(s, d_x, d_de)
    torch.cuda.synchronize()
    got = to_host(d_x)
    assert same_bytes(got[:n], want_x) and np.all(got[n:] == 0x3C)
    for a, b in zip(d_de, want_de):
        assert same_bytes(to_host(a), b)
    g.destroy()
    s.destroy()


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("flag", [K.KVL_TOKENS_APPEND, K.KVL_TOKENS_ALL], ids=["append", "all"])
def test_token_ranges(name, make, flag):
    w = make()
    if name == "cfg1":
        w.app[:] = [7, 16, 0, 25]                   # cfg1 has no tail of its own; 4 x 63 blocks cover 1008 tokens
        w.hit[:] = [1000, 992, 1001, 983]
    run_range_hop(w, flag)
    run_range_hop(w, flag, unit_bytes=2048, variant=2)


PIPE_VARIANTS = [1 + (256 | 2 | n << 2 | sp << 3 | na << 6) for n in (0, 1) for sp in range(4) for na in (0, 1)]


@pytest.mark.parametrize("variant", list(range(129)) + [1 + (128 | n << 2 | sp << 3) for n in (0, 1) for sp in range(4)]
                         + PIPE_VARIANTS)
@pytest.mark.parametrize("threads", [64, 256, 1024])
def test_every_variant(variant, threads):
    # units of 5 KiB against 64..1024 threads x 4..8 vectors: full steps, ragged tails and idle lanes
    w = W.config(3, n_requests=6, token_scale=1 / 64)
    run_hop(w, layer=variant % 3, variant=variant, block_threads=threads, unit_bytes=5 * 1152)


@pytest.mark.parametrize("unit_bytes", [1152, 16 * 1152, 64 * 1152, 1 << 20])
def test_unit_sizes(unit_bytes):
    w = W.tiny(207, 10, 64, (1152,), 400, 1500, kind="runs")
    run_hop(w, unit_bytes=unit_bytes)
    run_hop(w, unit_bytes=unit_bytes, variant=2)
    run_hop(w, unit_bytes=unit_bytes, variant=3, block_threads=64)
    run_hop(w, unit_bytes=unit_bytes, variant=4)


@pytest.mark.parametrize("seed", range(64))
def test_random_batches(seed):
    """Random small batches: all table kinds, ragged hits, 1-3 planes, rows that take the vector
    path with and without line alignment and rows that take the byte path."""
    rng = np.random.Generator(np.random.PCG64(7000 + seed))
    bs = int(rng.choice([1, 2, 3, 8, 16, 64]))
    planes = int(rng.integers(1, 4))
    rows = tuple(int(rng.choice([5, 16, 36, 48, 656, 1152])) for _ in range(planes))
    kind = ["random", "fragmented", "contiguous", "runs"][seed % 4]
    R = int(rng.integers(1, 9))
    max_tokens = int(rng.integers(1, 40 * bs + 2))
    pool_blocks = R * (max_tokens // bs + 4) + 3
    w = W.tiny(7000 + seed, R, bs, rows, pool_blocks, max_tokens, kind=kind)
    ub = int(rng.choice([0, 700, 5000, 1 << 16]))
    run_hop(w, unit_bytes=ub)
    run_range_hop(w, K.KVL_TOKENS_APPEND, unit_bytes=ub)
    run_range_hop(w, K.KVL_TOKENS_ALL, unit_bytes=ub, block_threads=64)


@pytest.mark.parametrize("bs", [8, 32, 128, 256])
@pytest.mark.parametrize("row", [64, 656, 2048, 16384])
def test_block_geometries(bs, row):
    """Block sizes from 512 bytes to 4 MiB under the default tuning: blocks far smaller than a
    tile, blocks that are split into several descriptors, rows with and without 128-byte alignment."""
    blocks_per_req = max(2, min(24, (6 << 20) // (bs * row)))
    w = W.tiny(300 + bs + row, 5, bs, (row,), 5 * (blocks_per_req + 3) + 7, bs * blocks_per_req, kind="runs")
    run_hop(w)
    run_range_hop(w, K.KVL_TOKENS_ALL)


def test_layers_are_independent_pools():
    w = W.config(1)
    for layer in range(w.layout.n_layers):
        run_hop(w, layer=layer)


def test_nan_and_inf_patterns_survive():
    w = W.tiny(208, 3, 16, (32,), 16, 60)
    bs, rows = 16, (32,)
    pool = np.zeros(16 * 16 * 32, dtype=np.uint8)
    v = pool.view(np.uint16)
    v[0::4], v[1::4], v[2::4], v[3::4] = 0x7FC1, 0xFF80, 0x7F80, 0xFFFF     # bf16 NaN, -inf, +inf, NaN
    want = oracle.pack(bs, rows, w.hit, w.src.tables, [pool])
    g = dev_plan(w, "src", K.KVL_GATHER)
    d_x = torch.zeros(g.payload_bytes, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, [to_dev(pool)], d_x)
    assert same_bytes(to_host(d_x), want)


def test_empty_and_zero_hit_batches():
    lay = K.make_layout(1, 16, (32,), 8)
    pool = torch.full((8 * 16 * 32,), 7, dtype=torch.uint8, device="cuda")
    x = torch.full((64,), 9, dtype=torch.uint8, device="cuda")
    for hit, app, tabs in (([], [], []), ([0, 0], [0, 5], [np.zeros(0, np.int32), np.array([3], np.int32)])):
        g = K.kvl_plan(lay, hit, app, tabs, K.KVL_GATHER | K.KVL_SCATTER)
        assert g.payload_bytes == 0
        K.kvl_pack_layer(g, [pool], x)
        K.kvl_unpack_layer(g, x, [pool])
        torch.cuda.synchronize()
        assert torch.all(pool == 7) and torch.all(x == 9)


def test_errors_from_the_device_entry_points():
    w = W.tiny(209, 3, 16, (32,), 32, 60, allow_zero_hit=False)
    g = dev_plan(w, "src", K.KVL_GATHER)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    pool = [torch.zeros(32 * 16 * 32, dtype=torch.uint8, device="cuda")]
    small = torch.zeros(g.payload_bytes - 16, dtype=torch.uint8, device="cuda")
    full = torch.zeros(g.payload_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(K.KvlError) as e:
        K.kvl_pack_layer(g, pool, small)
    assert e.value.code == K.KVL_ESPACE
    with pytest.raises(K.KvlError) as e:
        K.kvl_unpack_layer(s, small, pool)
    assert e.value.code == K.KVL_ESPACE
    with pytest.raises(K.KvlError) as e:
        K.kvl_pack_layer(s, pool, full)            # scatter plan used to gather
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(K.KvlError) as e:
        K.kvl_unpack_layer(g, full, pool)          # gather plan used to scatter
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(ValueError):                # the binding knows the pool is too small
        K.kvl_pack_layer(g, [pool[0][:100]], full)


def test_misaligned_buffers_take_the_byte_path():
    w = W.tiny(210, 4, 16, (48,), 40, 100)
    bs, rows = 16, (48,)
    src = W.fill_pool(w, 0, "src")
    want = oracle.pack(bs, rows, w.hit, w.src.tables, src)
    g = dev_plan(w, "src", K.KVL_GATHER)
    big = torch.zeros(src[0].size + 16, dtype=torch.uint8, device="cuda")
    big[3:3 + src[0].size] = to_dev(src[0])
    xb = torch.zeros(want.size + 16, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, [big[3:3 + src[0].size]], xb[5:5 + want.size])
    assert same_bytes(to_host(xb[5:5 + want.size]), want)
    assert int(xb[:5].sum()) == 0 and int(xb[5 + want.size:].sum()) == 0


def test_non_default_stream():
    w = W.config(1)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool(w, 1, "src")
    want = oracle.pack(bs, rows, w.hit, w.src.tables, src)
    g = dev_plan(w, "src", K.KVL_GATHER)
    d_src = planes_to_dev(src)
    d_x = torch.zeros(g.payload_bytes, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    K.kvl_pack_layer(g, d_src, d_x, stream=st)
    st.synchronize()
    assert same_bytes(to_host(d_x), want)


def test_copy_linear():
    a = to_dev(np.random.Generator(np.random.PCG64(1)).integers(0, 256, size=(1 << 20) + 4096 + 16, dtype=np.uint8))
    b = torch.zeros_like(a)
    K.kvl_copy_linear(a, b)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# --------------------------------------------------------------------------
# host buffer -> HBM
# --------------------------------------------------------------------------

H2D_CASES = [c for c in CASES if c[0] in ("tiny-runs-2planes", "tiny-oddrow", "cfg1", "cfg2-small", "cfg4-small")]


@pytest.mark.parametrize("name,make", H2D_CASES, ids=[c[0] for c in H2D_CASES])
@pytest.mark.parametrize("chunk_kb,slots", [(64, 1), (64, 3), (1024, 2), (16, 8), (16, 12), (0, 0)])
def test_h2d_unpack(name, make, chunk_kb, slots):
    w = make()
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    n = oracle.payload_bytes(w.hit, rows)
    x = W.random_payload(w, 0, n)
    want = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, x, want)
    s = dev_plan(w, "dst", K.KVL_SCATTER, unit_bytes=16384)
    host = pinned_from(x)
    chunk = chunk_kb * 1024
    staging = torch.zeros(chunk * slots, dtype=torch.uint8, device="cuda") if chunk else None   # 0: zero copy
    d_dst = planes_to_dev(W.sentinel_pool(w, "dst"))
    torch.cuda.synchronize()
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    K.kvl_h2d_unpack_layer(s, host, staging, chunk, d_dst, cs, ks)
    # a second layer through the same staging ring, queued at once
    x2 = W.random_payload(w, 1, n)
    host2 = pinned_from(x2)
    d_dst2 = planes_to_dev(W.sentinel_pool(w, "dst"))
    K.kvl_h2d_unpack_layer(s, host2, staging, chunk, d_dst2, cs, ks)
    ks.synchronize()
    cs.synchronize()
    for a, b in zip(d_dst, want):
        assert same_bytes(to_host(a), b)
    want2 = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, x2, want2)
    for a, b in zip(d_dst2, want2):
        assert same_bytes(to_host(a), b)


@pytest.mark.parametrize("name,make", H2D_CASES[:4], ids=[c[0] for c in H2D_CASES[:4]])
def test_h2d_zero_copy_and_blockwise(name, make):
    """Two other ways from the pinned host buffer into the pool: the scatter kernel reading
    host memory itself, and one copy-engine copy per descriptor."""
    w = make()
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    n = oracle.payload_bytes(w.hit, rows)
    x = W.random_payload(w, 3, n)
    want = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, x, want)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    host = pinned_from(x)
    a = planes_to_dev(W.sentinel_pool(w, "dst"))
    b = planes_to_dev(W.sentinel_pool(w, "dst"))
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    K.kvl_unpack_layer(s, host, a, stream=st)
    copies = K.kvl_h2d_blockwise_layer(s, host, b, stream=st)
    st.synchronize()
    assert copies == s.n_units * len(rows)
    for got_a, got_b, ref in zip(a, b, want):
        assert same_bytes(to_host(got_a), ref) and same_bytes(to_host(got_b), ref)
    # the same copies submitted as one batch, where the loaded HIP runtime has the call
    c = planes_to_dev(W.sentinel_pool(w, "dst"))
    torch.cuda.synchronize()
    try:
        copies = K.kvl_h2d_blockwise_batched_layer(s, host, c, stream=st)
    except K.KvlError as e:
        assert e.code == K.KVL_ENOSYS
    else:
        st.synchronize()
        assert copies == s.n_units * len(rows)
        for got_c, ref in zip(c, want):
            assert same_bytes(to_host(got_c), ref)


FB_CASES = [c for c in CASES if c[0] in ("tiny-random", "tiny-runs-2planes", "tiny-oddrow", "tiny-3planes",
                                         "cfg2-small", "cfg4-small")]


@pytest.mark.parametrize("name,make", FB_CASES, ids=[c[0] for c in FB_CASES])
@pytest.mark.parametrize("where", ["device", "pinned"])
@pytest.mark.parametrize("flag", [0, K.KVL_TOKENS_ALL], ids=["hit", "all"])
def test_full_block_layout(name, make, where, flag):
    """Decode pool -> Full Blocks (persist), then Full Blocks -> prefill pool (load), layer by
    layer, against the oracle's storage-layout functions."""
    w = make()
    L = 3
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    zero = np.zeros_like(w.hit)
    first, count = (zero, w.hit) if flag == 0 else (zero, w.hit + w.app)
    g = K.kvl_plan(K.make_layout(L, bs, rows, w.src.pool_blocks), w.hit, w.app, w.src.tables,
                   K.KVL_GATHER | K.KVL_NO_MERGE | flag)
    s = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                   K.KVL_SCATTER | K.KVL_NO_MERGE | flag, unit_bytes=8192)
    fb, nfb = g.fullblock_geometry()
    assert (fb, nfb) == s.fullblock_geometry()
    nbytes = max(16, fb * nfb)
    want_buf = np.full(nbytes + 64, 0x5A, dtype=np.uint8)
    if where == "device":
        buf = torch.full((nbytes + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    else:
        buf = torch.full((nbytes + 64,), 0x5A, dtype=torch.uint8).pin_memory()
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    srcs = []
    for l in range(L):
        pools = W.fill_pool(w, l, "src")
        oracle.pool_to_fullblocks(bs, L, rows, first, count, w.src.tables, l, pools, want_buf)
        srcs.append(planes_to_dev(pools))
        torch.cuda.synchronize()
        K.kvl_pool_to_fullblocks_layer(g, srcs[l], l, buf, stream=st)
    st.synchronize()
    got_buf = to_host(buf) if where == "device" else buf.numpy()
    assert same_bytes(got_buf, want_buf), "Full-Block buffer differs from the oracle"
    # the same persist staged through HBM (kernel into a slot, runtime copies out), 2 Layer Blocks per chunk
    if fb * nfb:
        buf2 = torch.full((nbytes + 64,), 0x5A, dtype=torch.uint8, device="cuda") if where == "device" else \
            torch.full((nbytes + 64,), 0x5A, dtype=torch.uint8).pin_memory()
        chunk = -(-2 * (fb // L) // 16) * 16
        staging = torch.zeros(3 * chunk, dtype=torch.uint8, device="cuda")
        cs2 = torch.cuda.Stream()
        torch.cuda.synchronize()
        for l in range(L):
            K.kvl_d2h_fullblocks_layer(g, srcs[l], l, staging, chunk, buf2, st, cs2)
        st.synchronize()
        cs2.synchronize()
        got2 = to_host(buf2) if where == "device" else buf2.numpy()
        assert same_bytes(got2, want_buf), "staged Full-Block buffer differs from the oracle"
    for l in (L - 1, 0):
        want = W.sentinel_pool(w, "dst")
        oracle.fullblocks_to_pool(bs, L, rows, first, count, w.dst.tables, l, want_buf, want)
        got = planes_to_dev(W.sentinel_pool(w, "dst"))
        torch.cuda.synchronize()
        K.kvl_fullblocks_to_pool_layer(s, buf, l, got, stream=st)
        st.synchronize()
        for a, b in zip(got, want):
            assert same_bytes(to_host(a), b), f"layer {l} loaded from Full Blocks differs from the oracle"
        # the same load staged through HBM by strided copies: 1 or 3 Layer Blocks per chunk, 1 or 2 slots
        lb = fb // L
        for blocks_per_chunk, n_slots in ((1, 1), (3, 2)):
            chunk = -(-blocks_per_chunk * lb // 16) * 16
            staging = torch.zeros(n_slots * chunk, dtype=torch.uint8, device="cuda")
            got = planes_to_dev(W.sentinel_pool(w, "dst"))
            cs = torch.cuda.Stream()
            torch.cuda.synchronize()
            K.kvl_h2d_fullblocks_layer(s, buf, l, staging, chunk, got, cs, st)
            st.synchronize()
            cs.synchronize()
            for a, b in zip(got, want):
                assert same_bytes(to_host(a), b), f"layer {l} staged from Full Blocks differs from the oracle"
    if fb // L >= 32:
        tiny_stage = torch.zeros(max(16, (fb // L) // 2 // 16 * 16), dtype=torch.uint8, device="cuda")
        with pytest.raises(K.KvlError) as e:       # a chunk smaller than one Layer Block
            K.kvl_h2d_fullblocks_layer(s, buf, 0, tiny_stage, tiny_stage.numel(), planes_to_dev(W.sentinel_pool(w, "dst")),
                                       st, st)
        assert e.value.code == K.KVL_ESPACE
    # errors: merged plan, short buffer, layer out of range
    merged = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables, K.KVL_SCATTER | flag)
    pool = planes_to_dev(W.sentinel_pool(w, "dst"))
    with pytest.raises(K.KvlError) as e:
        K.kvl_fullblocks_to_pool_layer(merged, buf, 0, pool)
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(K.KvlError) as e:
        K.kvl_fullblocks_to_pool_layer(s, buf, L, pool)
    assert e.value.code == K.KVL_EINVAL
    if fb * nfb > 64:
        with pytest.raises(K.KvlError) as e:
            K.kvl_fullblocks_to_pool_layer(s, buf[:fb * nfb - 16], 0, pool)
        assert e.value.code == K.KVL_ESPACE


def test_h2d_errors():
    w = W.tiny(211, 3, 16, (32,), 32, 60, allow_zero_hit=False)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    host = torch.zeros(s.payload_bytes, dtype=torch.uint8, pin_memory=True)
    pool = [torch.zeros(32 * 16 * 32, dtype=torch.uint8, device="cuda")]
    staging = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    with pytest.raises(K.KvlError) as e:
        K.kvl_h2d_unpack_layer(s, host, staging, 1 << 17, pool, cs, ks)    # staging smaller than a chunk
    assert e.value.code == K.KVL_ESPACE
    with pytest.raises(K.KvlError) as e:
        K.kvl_h2d_unpack_layer(s, host, staging, 16, pool, cs, ks)         # chunk smaller than a descriptor
    assert e.value.code == K.KVL_ESPACE
    with pytest.raises(TypeError):
        K.kvl_h2d_unpack_layer(s, torch.zeros(s.payload_bytes, dtype=torch.uint8), staging, 1 << 16, pool, cs, ks)


# --------------------------------------------------------------------------
# layer-wise streaming
# --------------------------------------------------------------------------

@pytest.mark.parametrize("S", [1, 2, 3])
@pytest.mark.parametrize("H", [1, 2, 6])
@pytest.mark.parametrize("chunk", [8192, 0], ids=["staged", "zerocopy"])
def test_stream_layers_observables(S, H, chunk):
    L = 6
    w = W.tiny(212, 6, 16, (64, 32), 96, 200, n_layers=L)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    n = oracle.payload_bytes(w.hit, rows)
    payloads = [W.random_payload(w, l, n) for l in range(L)]
    # oracle: what the compute of each layer must see in its slot
    o_slots = [W.sentinel_pool(w, "dst", 0xEE) for _ in range(S)]
    o_host = [np.zeros(n, np.uint8) for _ in range(H)]
    want = []
    gen = oracle.stream_layers(bs, rows, w.hit, w.dst.tables, o_host, L, o_slots)
    for l in range(L):
        o_host[l % H][:] = payloads[l]
        _, s_idx, planes = next(gen)
        want.append([p.copy() for p in planes])

    s = dev_plan(w, "dst", K.KVL_SCATTER, unit_bytes=4096)
    host = [torch.zeros(n, dtype=torch.uint8, pin_memory=True) for _ in range(H)]
    slots = [planes_to_dev(W.sentinel_pool(w, "dst", 0xEE)) for _ in range(S)]
    snaps = [[torch.zeros_like(pl) for pl in slots[0]] for _ in range(L)]
    # probes: first 16 bytes of a few rows
    probes = [(0, 0), (1, 32 * 5), (0, 64 * 17)]
    probe_out = torch.zeros(L * len(probes) * 16, dtype=torch.uint8, device="cuda")
    staging = torch.zeros(3 * 8192, dtype=torch.uint8, device="cuda")
    filled = []

    def fill(layer, slot):
        host[slot].numpy()[:] = payloads[layer]
        filled.append((layer, slot))

    torch.cuda.synchronize()
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    st = K.kvl_stream_layers(s, host, slots, staging if chunk else None, chunk, 50, cs, ks, ms, n_layers=L, probes=probes,
                             probe_out=probe_out, snapshots=snaps, host_fill=fill, per_layer_times=True)
    assert filled == [(l, l % H) for l in range(L)]
    for l in range(L):
        for p in range(len(rows)):
            assert same_bytes(to_host(snaps[l][p]), want[l][p]), f"layer {l} plane {p}: compute saw the wrong cache"
    po = to_host(probe_out).reshape(L, len(probes), 16)
    for l in range(L):
        for i, (pl, off) in enumerate(probes):
            assert po[l, i].tobytes() == want[l][pl][off:off + 16].tobytes()
    # ordering on the device clock: compute(l) after load(l); compute takes >= 50 us; layers in order
    tl, tb, te = st["t_loaded"], st["t_compute_begin"], st["t_compute_end"]
    assert np.all(tb >= tl - 1e-3)
    assert np.all(te - tb >= 0.045)
    assert np.all(np.diff(tb) > 0)
    assert st["total_ms"] >= L * 0.05
    assert st["h2d_bytes"] == n * L


@pytest.mark.parametrize("S", [1, 2])
@pytest.mark.parametrize("where", ["device", "pinned", "pinned-staged"])
def test_stream_layers_from_full_blocks(S, where):
    """Layer-wise load straight from the storage layout: what each layer's compute sees."""
    L = 5
    w = W.tiny(213, 6, 16, (64, 32), 96, 200, n_layers=L)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    zero = np.zeros_like(w.hit)
    nfb, fb = oracle.fullblock_count(bs, zero, w.hit), oracle.fullblock_bytes(bs, L, rows)
    blocks = W.random_payload(w, 9, nfb * fb)
    o_slots = [W.sentinel_pool(w, "dst", 0xEE) for _ in range(S)]
    want = []
    for _, _, planes in oracle.stream_layers_fullblocks(bs, L, rows, zero, w.hit, w.dst.tables, blocks, o_slots):
        want.append([p.copy() for p in planes])
    s = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                   K.KVL_SCATTER | K.KVL_NO_MERGE)
    assert s.fullblock_geometry() == (fb, nfb)
    buf = to_dev(blocks) if where == "device" else pinned_from(blocks)
    slots = [planes_to_dev(W.sentinel_pool(w, "dst", 0xEE)) for _ in range(S)]
    snaps = [[torch.zeros_like(pl) for pl in slots[0]] for _ in range(L)]
    # staged: strided copies bring 5 Layer Blocks at a time into each of 3 staging slots
    chunk = 5 * (fb // L) if where == "pinned-staged" else 0
    staging = torch.zeros(3 * chunk, dtype=torch.uint8, device="cuda") if chunk else None
    torch.cuda.synchronize()
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    st = K.kvl_stream_layers(s, None, slots, staging, chunk, 50, cs, ks, ms, n_layers=L, snapshots=snaps,
                             per_layer_times=True, full_blocks=buf)
    for l in range(L):
        for p in range(len(rows)):
            assert same_bytes(to_host(snaps[l][p]), want[l][p]), f"layer {l} plane {p}"
    assert np.all(st["t_compute_begin"] >= st["t_loaded"] - 1e-3)
    merged = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
    with pytest.raises(K.KvlError) as e:
        K.kvl_stream_layers(merged, None, slots, None, 0, 50, cs, ks, ms, n_layers=L, full_blocks=buf)
    assert e.value.code == K.KVL_EINVAL


def test_hip_graph_capture_and_replay():
    """pack and unpack only launch kernels, so a caller may capture them in a HIP graph (the
    launch-bound regime of small payloads).  Every replay, with fresh inputs and eager work in
    between, must equal the oracle."""
    w = W.config(1)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    g = dev_plan(w, "src", K.KVL_GATHER)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    n = g.payload_bytes
    src = [planes_to_dev(W.fill_pool(w, l, "src")) for l in range(L)]
    dst = [planes_to_dev(W.sentinel_pool(w, "dst")) for l in range(L)]
    x = [torch.zeros(n, dtype=torch.uint8, device="cuda") for _ in range(L)]
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(graph, stream=st):
            for l in range(L):
                K.kvl_pack_layer(g, src[l], x[l], stream=st)
                K.kvl_unpack_layer(s, x[l], dst[l], stream=st)
    for rep in range(3):
        fills = [W.fill_pool(w, 10 * rep + l, "src") for l in range(L)]
        for l in range(L):
            src[l][0].copy_(to_dev(fills[l][0]))          # eager work between replays
            dst[l][0].fill_(0xA5)
            x[l].zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            graph.replay()
        st.synchronize()
        for l in range(L):
            want_x = oracle.pack(bs, rows, w.hit, w.src.tables, fills[l])
            want = W.sentinel_pool(w, "dst")
            oracle.unpack(bs, rows, w.hit, w.dst.tables, want_x, want)
            assert same_bytes(to_host(x[l]), want_x), f"replay {rep} layer {l}: transfer buffer"
            assert same_bytes(to_host(dst[l][0]), want[0]), f"replay {rep} layer {l}: pool"


@pytest.mark.parametrize("chunk", [1 << 20, 0], ids=["staged", "zerocopy"])
def test_hip_graph_capture_of_the_host_buffer_load(chunk):
    """The host-buffer load forks onto the library's lanes and joins again, all by events, so a
    caller may capture it too (both stream arguments the capturing stream; the lanes are made
    by an eager call first).  Every replay, with a fresh host buffer and eager work in between,
    must equal the oracle."""
    w = W.config(1)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    n = s.payload_bytes
    host = torch.zeros(n, dtype=torch.uint8, pin_memory=True)
    staging = torch.zeros(2 * chunk, dtype=torch.uint8, device="cuda") if chunk else None
    dst = planes_to_dev(W.sentinel_pool(w, "dst"))
    st = torch.cuda.Stream()
    torch.cuda.synchronize()
    K.kvl_h2d_unpack_layer(s, host, staging, chunk, dst, st, st)       # eager: creates the lanes
    st.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(st):
        with torch.cuda.graph(graph, stream=st):
            K.kvl_h2d_unpack_layer(s, host, staging, chunk, dst, st, st)
    for rep in range(3):
        x = W.random_payload(w, 20 + rep, n)
        host.numpy()[:] = x
        for d in dst:
            d.fill_(0xA5)                                              # eager work between replays
        torch.cuda.synchronize()
        with torch.cuda.stream(st):
            graph.replay()
        st.synchronize()
        want = W.sentinel_pool(w, "dst")
        oracle.unpack(bs, rows, w.hit, w.dst.tables, x, want)
        for a, b in zip(dst, want):
            assert same_bytes(to_host(a), b), f"replay {rep}"


@pytest.mark.parametrize("name,make", H2D_CASES, ids=[c[0] for c in H2D_CASES])
def test_host_buffers_both_ways_whole_prompt(name, make):
    """The prefill-engine read path after a layer's compute (Section 4.1, steps 5-9): hit and miss
    rows together go to the decode engine's host buffer (pack straight into pinned memory), and
    from there into the decode engine's HBM (host-buffer load of the whole prompt)."""
    w = make()
    if name == "cfg1":
        w.hit[:] = [1000, 992, 1001, 983]
        w.app[:] = [7, 16, 0, 25]
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    zero, tot = np.zeros_like(w.hit), w.hit + w.app
    pe = W.fill_pool(w, 2, "dst")
    want_x = oracle.pack_range(bs, rows, zero, tot, w.dst.tables, pe)
    want_de = W.sentinel_pool(w, "src")
    oracle.unpack_range(bs, rows, zero, tot, w.src.tables, want_x, want_de)
    g = K.kvl_plan(K.make_layout(1, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                   K.KVL_GATHER | K.KVL_TOKENS_ALL)
    s = K.kvl_plan(K.make_layout(1, bs, rows, w.src.pool_blocks), w.hit, w.app, w.src.tables,
                   K.KVL_SCATTER | K.KVL_TOKENS_ALL, unit_bytes=16384)
    n = g.payload_bytes
    host = torch.full((n + 64,), 0x3C, dtype=torch.uint8).pin_memory()
    d_pe = planes_to_dev(pe)
    d_de = planes_to_dev(W.sentinel_pool(w, "src"))
    staging = torch.zeros(3 * 65536, dtype=torch.uint8, device="cuda")
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    K.kvl_pack_layer(g, d_pe, host, stream=ks)
    ks.synchronize()
    got = host.numpy()
    assert same_bytes(got[:n], want_x) and np.all(got[n:] == 0x3C)
    K.kvl_h2d_unpack_layer(s, host, staging, 65536, d_de, cs, ks)
    ks.synchronize()
    for a, b in zip(d_de, want_de):
        assert same_bytes(to_host(a), b)


def test_stream_layers_argument_errors():
    w = W.tiny(215, 3, 16, (32,), 32, 60, allow_zero_hit=False)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    g = dev_plan(w, "dst", K.KVL_GATHER)
    n = s.payload_bytes
    host = [torch.zeros(n, dtype=torch.uint8, pin_memory=True)]
    slots = [[torch.zeros(32 * 16 * 32, dtype=torch.uint8, device="cuda")]]
    staging = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    out = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()

    def call(plan=s, **kw):
        args = dict(host_layers=host, dev_slots=slots, dev_staging=staging, chunk_bytes=1 << 16, compute_us=10,
                    copy_stream=cs, kernel_stream=ks, compute_stream=ms, n_layers=2)
        args.update(kw)
        return K.kvl_stream_layers(plan, **args)

    assert call()["h2d_bytes"] == 2 * n                                   # the well-formed call works
    for bad in (dict(compute_us=2_000_000),                               # absurd compute time
                dict(probes=[(0, 8)], probe_out=out),                     # probe not 16-byte aligned
                dict(probes=[(1, 0)], probe_out=out),                     # plane out of range
                dict(probes=[(0, 32 * 16 * 32)], probe_out=out),          # probe beyond the slot
                dict(chunk_bytes=16),                                     # chunk smaller than a descriptor
                dict(plan=g)):                                            # gather plan
        with pytest.raises(K.KvlError) as e:
            call(**bad)
        assert e.value.code in (K.KVL_EINVAL, K.KVL_ESPACE), bad
    with pytest.raises(K.KvlError):
        call(dev_slots=[])                                                # no destination slot
    torch.cuda.synchronize()


def test_h2d_lanes_confined_to_a_few_compute_units():
    """A compute-unit mask on the library's lanes changes where the scatters run, not what they write."""
    w = W.config(2, n_requests=7, token_scale=1 / 32)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    n = oracle.payload_bytes(w.hit, rows)
    x = W.random_payload(w, 4, n)
    want = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, x, want)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    host = pinned_from(x)
    staging = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    for mask in (list(range(8)), None):
        s.set_lane_cu_mask(mask)
        got = planes_to_dev(W.sentinel_pool(w, "dst"))
        torch.cuda.synchronize()
        K.kvl_h2d_unpack_layer(s, host, staging, 1 << 20, got, cs, ks)
        ks.synchronize()
        for a, b in zip(got, want):
            assert same_bytes(to_host(a), b), f"mask {mask and len(mask)}"


def test_two_host_threads_with_their_own_plans():
    """Plans are per-thread objects; the library's shared state (descriptor cache, error slots)
    must stand two threads building, running and destroying plans at the same time."""
    import threading
    errors = []

    def worker(seed):
        try:
            w = W.tiny(400 + seed, 6, 16, (1152,), 256, 400, kind="random")
            bs, rows = w.layout.block_tokens, w.layout.row_bytes
            src = W.fill_pool(w, seed, "src")
            want_x = oracle.pack(bs, rows, w.hit, w.src.tables, src)
            want = W.sentinel_pool(w, "dst")
            oracle.unpack(bs, rows, w.hit, w.dst.tables, want_x, want)
            d_src = planes_to_dev(src)
            st = torch.cuda.Stream()
            for _ in range(25):
                g = dev_plan(w, "src", K.KVL_GATHER)
                s = dev_plan(w, "dst", K.KVL_SCATTER)
                x = torch.zeros(g.payload_bytes, dtype=torch.uint8, device="cuda")
                d = planes_to_dev(W.sentinel_pool(w, "dst"))
                torch.cuda.current_stream().synchronize()
                K.kvl_pack_layer(g, d_src, x, stream=st)
                K.kvl_unpack_layer(s, x, d, stream=st)
                st.synchronize()
                assert same_bytes(to_host(x), want_x) and same_bytes(to_host(d[0]), want[0])
                g.destroy()
                s.destroy()
        except Exception as e:  # noqa: BLE001
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors


@pytest.mark.parametrize("name,make", CASES, ids=[c[0] for c in CASES])
def test_fused_move_equals_pack_then_unpack(name, make):
    """Pool to pool in one kernel: the destination must be what pack followed by unpack leaves."""
    w = make()
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool(w, 3, "src")
    want = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, oracle.pack(bs, rows, w.hit, w.src.tables, src), want)
    g = dev_plan(w, "src", K.KVL_GATHER)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    m = K.kvl_plan_pair(g, s)
    g.destroy()
    s.destroy()                                   # the paired plan stands on its own
    d_src = planes_to_dev(src)
    d_dst = planes_to_dev(W.sentinel_pool(w, "dst"))
    K.kvl_move_layer(m, d_src, d_dst)
    torch.cuda.synchronize()
    for a, b in zip(d_dst, want):
        assert same_bytes(to_host(a), b)
    for a, b in zip(d_src, src):
        assert same_bytes(to_host(a), b)
    x = torch.zeros(max(16, m.payload_bytes), dtype=torch.uint8, device="cuda")
    with pytest.raises(K.KvlError) as e:
        K.kvl_pack_layer(m, d_src, x)             # a paired plan only moves
    assert e.value.code == K.KVL_EINVAL


@pytest.mark.parametrize("name,make", [c for c in CASES if c[0] in ("tiny-random", "tiny-3planes", "cfg1", "cfg2-small",
                                                                     "cfg4-small", "trace32k-6req")],
                         ids=lambda v: v if isinstance(v, str) else "")
def test_pipelined_walk_on_every_kind_of_batch(name, make):
    """The pipelined form has a main loop over the trips every workgroup shares and a tail of up
    to three tiles: batches of a few tiles (no loop at all), of a few trips, ragged descriptors,
    several planes, 656-byte rows (aligned first tiles)."""
    w = make()
    for threads in (64, 256):
        run_hop(w, variant=PIPE_VARIANTS[5], block_threads=threads)
        run_hop(w, variant=PIPE_VARIANTS[-1], block_threads=threads, max_groups=3)    # three workgroups walk it all
        run_hop(w, variant=PIPE_VARIANTS[2], block_threads=threads, unit_bytes=4096, max_groups=7)


def test_flat_kernel_split_over_several_launches():
    """Token-granular pools: the flat kernel numbers its lanes with 32 bits and spreads the
    descriptors over several launches when they would not fit.  max_groups lowers the
    workgroups per launch, so that a small batch takes the same path: 3 and more launches,
    the last one ragged."""
    for make in (lambda: W.tiny(215, 9, 1, (1152,), 3000, 300),
                 lambda: W.tiny(216, 7, 2, (256, 64), 2000, 250, kind="fragmented")):
        w = make()
        g = dev_plan(w, "src", K.KVL_GATHER)
        n_units = g.n_units
        g.destroy()
        vecs = max(w.layout.row_bytes) // 16 * w.layout.block_tokens          # lanes per descriptor
        for launches in (3, 7):
            per_launch = -(-n_units // launches)                               # descriptors per launch
            groups = max(1, per_launch * vecs // 256)
            assert -(-n_units // max(1, groups * 256 // vecs)) >= launches
            run_hop(w, max_groups=groups)                                      # default (flat) kernels, capped
            run_hop(w, variant=1 + (128 | 4 | 8), max_groups=groups)           # an explicit flat variant


def test_destroying_a_plan_does_not_wait_for_the_device():
    """kvl_plan_destroy retires the descriptor array behind events instead of synchronising: it
    returns at once while another stream is busy for a long time, and the array is not handed to
    the next plan while a kernel of the destroyed one has yet to run."""
    import time
    w = W.config(3, n_requests=12, token_scale=1 / 16)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool(w, 0, "src")
    want_x = oracle.pack(bs, rows, w.hit, w.src.tables, src, threads=8)
    d_src = planes_to_dev(src)
    busy, side = torch.cuda.Stream(), torch.cuda.Stream()
    # a kernel that spins for about 0.2 s: the counter torch's _sleep reads ticks at a rate found by trying
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda._sleep(1000)
    torch.cuda.synchronize()
    e0.record()
    torch.cuda._sleep(1_000_000)
    e1.record()
    e1.synchronize()
    spin_cycles = int(1_000_000 * 200.0 / max(e0.elapsed_time(e1), 1e-3))
    K.kvl_release_cached_memory()
    # (1) a long kernel on another stream: destroy returns while it is still running
    g = dev_plan(w, "src", K.KVL_GATHER)
    x = torch.zeros(g.payload_bytes, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, d_src, x, stream=side)
    side.synchronize()
    done = torch.cuda.Event()
    with torch.cuda.stream(busy):
        torch.cuda._sleep(spin_cycles)
        done.record(busy)
    t0 = time.perf_counter()
    g.destroy()
    dt = time.perf_counter() - t0
    still_running = not done.query()
    assert still_running, "the spinning kernel ended before the check: make it longer"
    assert dt < 5e-3, f"kvl_plan_destroy took {dt * 1e3:.1f} ms beside a busy stream"
    assert same_bytes(to_host(x), want_x)
    # (2) the plan's own kernel is still queued behind a long one when the plan goes; plans made
    # right after must not get its descriptor array (their descriptors differ)
    g = dev_plan(w, "src", K.KVL_GATHER)
    x.zero_()
    y = torch.zeros_like(x)
    torch.cuda.synchronize()                      # the fills above ran on the default stream
    with torch.cuda.stream(side):
        torch.cuda._sleep(spin_cycles)
    K.kvl_pack_layer(g, d_src, x, stream=side)
    g.destroy()
    other = W.config(3, n_requests=12, token_scale=1 / 16)
    other.src.tables = [t[::-1].copy() for t in other.src.tables]       # same sizes, other descriptors
    plans = [dev_plan(other, "src", K.KVL_GATHER) for _ in range(4)]
    K.kvl_pack_layer(plans[0], d_src, y, stream=busy)
    torch.cuda.synchronize()
    assert same_bytes(to_host(x), want_x), "a retired descriptor array was reused before its kernel had run"
    want_y = oracle.pack(bs, rows, other.hit, other.src.tables, src, threads=8)
    assert same_bytes(to_host(y), want_y)
    for p in plans:
        p.destroy()
    # (3) once the work is done the array does come back: no device memory is lost over many plans
    torch.cuda.synchronize()
    K.kvl_release_cached_memory()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(200):
        p = dev_plan(w, "src", K.KVL_GATHER)
        K.kvl_pack_layer(p, d_src, x, stream=side)
        p.destroy()                                                 # no synchronisation in between
    torch.cuda.synchronize()
    K.kvl_release_cached_memory()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < (8 << 20), f"{(free0 - free1) >> 20} MiB of device memory gone"


def test_plans_whose_caller_answers_for_their_lifetime():
    """KVL_CALLER_SYNCS: no event after each launch, the descriptor array goes back at once."""
    w = W.config(3, n_requests=12, token_scale=1 / 16)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool(w, 1, "src")
    want_x = oracle.pack(bs, rows, w.hit, w.src.tables, src, threads=8)
    want_dst = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, want_x, want_dst, threads=8)
    d_src = planes_to_dev(src)
    for _ in range(3):
        g = dev_plan(w, "src", K.KVL_GATHER | K.KVL_CALLER_SYNCS)
        s = dev_plan(w, "dst", K.KVL_SCATTER | K.KVL_CALLER_SYNCS)
        m = K.kvl_plan_pair(g, s)
        x = torch.zeros(g.payload_bytes, dtype=torch.uint8, device="cuda")
        d_dst = planes_to_dev(W.sentinel_pool(w, "dst"))
        d_dst2 = planes_to_dev(W.sentinel_pool(w, "dst"))
        K.kvl_pack_layer(g, d_src, x)
        K.kvl_unpack_layer(s, x, d_dst)
        K.kvl_move_layer(m, d_src, d_dst2)
        torch.cuda.synchronize()                       # the promise the flag makes
        for p in (g, s, m):
            p.destroy()
        assert same_bytes(to_host(x), want_x)
        for a, b, c in zip(d_dst, d_dst2, want_dst):
            assert same_bytes(to_host(a), c) and same_bytes(to_host(b), c)


def test_ceiling_kernels_stay_inside_their_buffers():
    """The reference streams of the benchmark: the copy modes move what they say, and nothing is
    written outside the bytes they were given."""
    block, k_dense, k_hop, skew = 64 * 656, 6, 7, 16
    payload = (1 << k_dense) * block
    guard = 4096
    hop = torch.randint(0, 255, ((1 << k_hop) * block + guard,), dtype=torch.uint8, device="cuda")
    dense = torch.full((payload + 128 + guard,), 0x3C, dtype=torch.uint8, device="cuda")
    hop0 = hop.clone()
    table = ((torch.arange(1 << k_dense, dtype=torch.int64, device="cuda") * 0x9e3779b1) & ((1 << k_hop) - 1)).to(torch.int32)
    for tab in (None, table):
        dense.fill_(0x3C)
        K.kvl_ceiling_kernel(K.KVL_CEILING_COPY, hop[:(1 << k_hop) * block], dense[:payload + 128], payload,
                             block_bytes=block, hopping_side=0, skew_bytes=skew, hop_blocks_log2=k_hop, block_table=tab)
        torch.cuda.synchronize()
        got = to_host(dense)
        h = to_host(hop0)
        assert np.all(got[:skew] == 0x3C) and np.all(got[skew + payload:] == 0x3C)
        for u in (0, 1, 17, (1 << k_dense) - 1):
            b = (u * 0x9e3779b1) & ((1 << k_hop) - 1)
            assert got[skew + u * block: skew + (u + 1) * block].tobytes() == h[b * block:(b + 1) * block].tobytes()
    # the scatter direction writes only inside the hopping side's blocks; read-only writes nothing
    K.kvl_ceiling_kernel(K.KVL_CEILING_READ, dense[:payload + 128], hop[:(1 << k_hop) * block], payload,
                         block_bytes=block, hopping_side=1, skew_bytes=skew, hop_blocks_log2=k_hop)
    torch.cuda.synchronize()
    assert torch.equal(hop, hop0)
    K.kvl_ceiling_kernel(K.KVL_CEILING_COPY, dense[:payload + 128], hop[:(1 << k_hop) * block], payload,
                         block_bytes=block, hopping_side=1, skew_bytes=skew, hop_blocks_log2=k_hop, block_table=table)
    torch.cuda.synchronize()
    assert torch.equal(hop[(1 << k_hop) * block:], hop0[(1 << k_hop) * block:])
    d = to_host(dense)
    hh = to_host(hop)
    for u in (0, 5, (1 << k_dense) - 1):
        b = (u * 0x9e3779b1) & ((1 << k_hop) - 1)
        assert hh[b * block:(b + 1) * block].tobytes() == d[skew + u * block: skew + (u + 1) * block].tobytes()
    # linear modes
    n = 1 << 20
    a = torch.randint(0, 255, (n + 128,), dtype=torch.uint8, device="cuda")
    b = torch.full((n + guard,), 0x3C, dtype=torch.uint8, device="cuda")
    K.kvl_ceiling_kernel(K.KVL_CEILING_COPY, a, b[:n], n, skew_bytes=16)
    torch.cuda.synchronize()
    assert torch.equal(b[:n], a[16:16 + n]) and bool(torch.all(b[n:] == 0x3C))
    K.kvl_ceiling_kernel(K.KVL_CEILING_WRITE, a, b[:n], n)
    K.kvl_ceiling_kernel(K.KVL_CEILING_READ, a, b[:n], n)
    torch.cuda.synchronize()
    assert bool(torch.all(b[n:] == 0x3C))
    with pytest.raises(K.KvlError) as e:
        K.kvl_ceiling_kernel(K.KVL_CEILING_COPY, a, b[:n], 2 * n)
    assert e.value.code == K.KVL_ESPACE


def test_plans_do_not_leak_device_memory():
    w = W.config(3, n_requests=12, token_scale=1 / 16)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    host = torch.zeros(oracle.payload_bytes(w.hit, rows), dtype=torch.uint8, pin_memory=True)
    pool = planes_to_dev(W.sentinel_pool(w, "dst"))
    staging = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()

    def cycle():
        s = dev_plan(w, "dst", K.KVL_SCATTER, unit_bytes=16384)
        K.kvl_h2d_unpack_layer(s, host, staging, 1 << 20, pool, cs, ks)      # creates the plan's lanes
        ks.synchronize()
        s.destroy()

    for _ in range(20):
        cycle()
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(300):
        cycle()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < (8 << 20), f"{(free0 - free1) >> 20} MiB of device memory gone after 300 plans"
    K.kvl_release_cached_memory()


def test_check_buffer_classifies_pointers():
    dev = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    pinned = torch.zeros(1 << 16, dtype=torch.uint8, pin_memory=True)
    pageable = np.zeros(1 << 16, dtype=np.uint8)
    assert K.kvl_check_buffer(dev.data_ptr(), 1 << 20) == K.KVL_OK
    assert K.kvl_check_buffer(dev.data_ptr() + 4096, (1 << 20) - 4096) == K.KVL_OK
    assert K.kvl_check_buffer(dev.data_ptr(), 1 << 46) == K.KVL_ESPACE       # past any allocation's end
    assert K.kvl_check_buffer(pinned.data_ptr(), 1 << 16, allow_host=True) == K.KVL_OK
    assert K.kvl_check_buffer(pinned.data_ptr(), 1 << 16, allow_host=False) == K.KVL_EINVAL
    assert K.kvl_check_buffer(pageable.ctypes.data, 1 << 16, allow_host=True) == K.KVL_EINVAL
    assert K.kvl_check_buffer(0, 0) == K.KVL_OK and K.kvl_check_buffer(0, 16) == K.KVL_EINVAL
    # the failed look-ups above must not leave a sticky HIP error behind
    torch.cuda.synchronize()
    assert int((dev + 1).sum()) == 1 << 20


def test_entry_points_refuse_memory_the_device_cannot_address():
    """Raw C-ABI calls (the Python layer would stop these earlier) with pageable host
    memory where device or pinned memory is required: an error code, no launch."""
    import ctypes as C
    lib = K.binding._lib
    w = W.tiny(260, 3, 16, (32,), 32, 60, allow_zero_hit=False)
    g = dev_plan(w, "src", K.KVL_GATHER)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    pool = torch.zeros(32 * 16 * 32, dtype=torch.uint8, device="cuda")
    xfer = torch.zeros(g.payload_bytes, dtype=torch.uint8, device="cuda")
    host_pool = np.zeros(32 * 16 * 32, dtype=np.uint8)
    host_xfer = np.zeros(g.payload_bytes, dtype=np.uint8)
    good, bad = (C.c_void_p * 1)(pool.data_ptr()), (C.c_void_p * 1)(host_pool.ctypes.data)
    n = C.c_uint64(g.payload_bytes)
    assert lib.kvl_pack_layer(g.handle, bad, C.c_void_p(xfer.data_ptr()), n, None) == K.KVL_EINVAL
    assert lib.kvl_pack_layer(g.handle, good, C.c_void_p(host_xfer.ctypes.data), n, None) == K.KVL_EINVAL
    assert lib.kvl_unpack_layer(s.handle, C.c_void_p(host_xfer.ctypes.data), n, good, None) == K.KVL_EINVAL
    assert lib.kvl_unpack_layer(s.handle, C.c_void_p(xfer.data_ptr()), n, bad, None) == K.KVL_EINVAL
    # a pool plane that is device memory but shorter than the layout says
    tail = (C.c_void_p * 1)(pool.data_ptr() + pool.numel() - 64)
    big = K.make_layout(1, 16, (32,), 1 << 27)     # a 64 GiB pool: past the end of what holds `pool`
    gb = K.kvl_plan(big, w.hit, w.app, w.src.tables, K.KVL_GATHER)
    assert lib.kvl_pack_layer(gb.handle, tail, C.c_void_p(xfer.data_ptr()), n, None) == K.KVL_ESPACE
    # the same calls pass once the memory is right, and a plan may opt out of the checks
    assert lib.kvl_pack_layer(g.handle, good, C.c_void_p(xfer.data_ptr()), n, None) == K.KVL_OK
    lay = K.make_layout(w.layout.n_layers, 16, (32,), 32)
    g2 = K.kvl_plan(lay, w.hit, w.app, w.src.tables, K.KVL_GATHER | K.KVL_NO_POINTER_CHECKS)
    assert lib.kvl_pack_layer(g2.handle, good, C.c_void_p(xfer.data_ptr()), n, None) == K.KVL_OK
    torch.cuda.synchronize()


@pytest.mark.parametrize("S", [1, 2])
@pytest.mark.parametrize("chunk", [8192, 0], ids=["staged", "zerocopy"])
def test_stream_layers_with_the_callers_own_compute(S, chunk):
    """The per-layer computation is the caller's: torch kernels enqueued from the callback
    on the compute stream must see, layer by layer, what the oracle says the slot holds."""
    L, H = 5, 2
    w = W.tiny(261, 5, 16, (64, 32), 96, 180, n_layers=L)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    n = oracle.payload_bytes(w.hit, rows)
    payloads = [W.random_payload(w, l, n) for l in range(L)]
    o_slots = [W.sentinel_pool(w, "dst", 0xEE) for _ in range(S)]
    o_host = [np.zeros(n, np.uint8) for _ in range(H)]
    want = []
    gen = oracle.stream_layers(bs, rows, w.hit, w.dst.tables, o_host, L, o_slots)
    for l in range(L):
        o_host[l % H][:] = payloads[l]
        _, _, planes = next(gen)
        want.append([p.copy() for p in planes])

    s = dev_plan(w, "dst", K.KVL_SCATTER, unit_bytes=4096)
    host = [torch.zeros(n, dtype=torch.uint8, pin_memory=True) for _ in range(H)]
    slots = [planes_to_dev(W.sentinel_pool(w, "dst", 0xEE)) for _ in range(S)]
    seen = [[torch.zeros_like(pl) for pl in slots[0]] for _ in range(L)]
    sums = torch.zeros(L, dtype=torch.int64, device="cuda")
    staging = torch.zeros(3 * 8192, dtype=torch.uint8, device="cuda")
    calls = []

    def fill(layer, slot):
        host[slot].numpy()[:] = payloads[layer]

    torch.cuda.synchronize()
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()

    def compute(layer, slot, stream_handle):
        calls.append((layer, slot))
        assert stream_handle == ms.cuda_stream
        with torch.cuda.stream(ms):
            for p in range(len(rows)):
                seen[layer][p].copy_(slots[slot][p])
            sums[layer] = slots[slot][0].sum(dtype=torch.int64)

    st = K.kvl_stream_layers(s, host, slots, staging if chunk else None, chunk, 0, cs, ks, ms, n_layers=L,
                             host_fill=fill, compute=compute, per_layer_times=True)
    assert calls == [(l, l % S) for l in range(L)]
    for l in range(L):
        for p in range(len(rows)):
            assert same_bytes(to_host(seen[l][p]), want[l][p]), f"layer {l} plane {p}"
        assert int(sums[l]) == int(want[l][0].astype(np.int64).sum())
    assert np.all(st["t_compute_begin"] >= st["t_loaded"] - 1e-3)
    assert st["exposed_ms"] <= st["total_ms"]

    # a callback that fails ends the run with an error, and nothing is left running
    def broken(layer, slot, stream_handle):
        if layer == 2:
            raise RuntimeError("planted")
    with pytest.raises(K.KvlError) as e:
        K.kvl_stream_layers(s, host, slots, staging if chunk else None, chunk, 0, cs, ks, ms, n_layers=L,
                            host_fill=fill, compute=broken)
    assert e.value.code == K.KVL_EINVAL
    torch.cuda.synchronize()
    # the synthetic kernel's probes make no sense with a caller's computation
    with pytest.raises(K.KvlError) as e:
        K.kvl_stream_layers(s, host, slots, staging if chunk else None, chunk, 0, cs, ks, ms, n_layers=L,
                            probes=[(0, 0)], probe_out=torch.zeros(L * 16, dtype=torch.uint8, device="cuda"),
                            compute=compute)
    assert e.value.code == K.KVL_EINVAL


@pytest.mark.parametrize("name,make", H2D_CASES, ids=[c[0] for c in H2D_CASES])
@pytest.mark.parametrize("chunk_kb,slots", [(64, 1), (64, 3), (1024, 2), (16, 8)])
def test_d2h_pack_staged(name, make, chunk_kb, slots):
    """The gather into a pinned host buffer, staged: pack kernels into HBM slots, copy engine out."""
    w = make()
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    g = dev_plan(w, "src", K.KVL_GATHER, unit_bytes=16384)
    n = g.payload_bytes
    chunk = chunk_kb * 1024
    staging = torch.zeros(chunk * slots, dtype=torch.uint8, device="cuda")
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    hosts, wants = [], []
    torch.cuda.synchronize()
    for layer in (0, 1):                      # two layers through the same slots, queued at once
        src = W.fill_pool(w, layer, "src")
        wants.append(oracle.pack(bs, rows, w.hit, w.src.tables, src))
        host = torch.full((n + 64,), 0x3C, dtype=torch.uint8).pin_memory()
        d_src = planes_to_dev(src)
        torch.cuda.synchronize()
        K.kvl_d2h_pack_layer(g, d_src, staging, chunk, host, ks, cs)
        hosts.append((host, d_src))
    ks.synchronize()
    cs.synchronize()
    for (host, _), want in zip(hosts, wants):
        got = host.numpy()
        assert same_bytes(got[:n], want), "staged gather into host memory differs from the oracle"
        assert np.all(got[n:] == 0x3C), "wrote past the payload"
    # a scatter plan, a chunk of 0 and a short host buffer are refused
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    d_src = hosts[0][1]
    with pytest.raises(K.KvlError) as e:
        K.kvl_d2h_pack_layer(s, planes_to_dev(W.sentinel_pool(w, "dst")), staging, chunk, hosts[0][0], ks, cs)
    assert e.value.code == K.KVL_EINVAL
    with pytest.raises(K.KvlError) as e:
        K.kvl_d2h_pack_layer(g, d_src, staging, 0, hosts[0][0], ks, cs)
    assert e.value.code == K.KVL_EINVAL
    if n > 16:
        short = torch.zeros(n - 16, dtype=torch.uint8).pin_memory()
        with pytest.raises(K.KvlError) as e:
            K.kvl_d2h_pack_layer(g, d_src, staging, chunk, short, ks, cs)
        assert e.value.code == K.KVL_ESPACE


@pytest.mark.parametrize("S,Ho", [(1, 1), (2, 1), (2, 3)])
@pytest.mark.parametrize("out_chunk", [8192, 0], ids=["out-staged", "out-zerocopy"])
@pytest.mark.parametrize("in_chunk", [8192, 0], ids=["in-staged", "in-zerocopy"])
def test_stream_layers_with_outflow(S, Ho, out_chunk, in_chunk):
    """The whole loop of layer-wise prefill: layer l+1 is loaded while layer l is computed and
    layer l-1 (hit and appended rows, as the compute left them) leaves for host memory.  The
    compute here adds 1 to every byte of the slot; the oracle does the same to its slots."""
    L, H = 5, 2
    w = W.tiny(262, 5, 16, (64, 32), 96, 180, n_layers=L)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    n = oracle.payload_bytes(w.hit, rows)
    total = (w.hit + w.app).astype(np.uint32)
    n_out = oracle.payload_bytes(total, rows)
    payloads = [W.random_payload(w, l, n) for l in range(L)]
    o_slots = [W.sentinel_pool(w, "dst", 0xEE) for _ in range(S)]
    o_host = [np.zeros(n, np.uint8) for _ in range(H)]
    want_out = []
    gen = oracle.stream_layers(bs, rows, w.hit, w.dst.tables, o_host, L, o_slots)
    for l in range(L):
        o_host[l % H][:] = payloads[l]
        _, s_idx, planes = next(gen)
        for p in planes:                       # the compute of layer l
            p += 1
        want_out.append(oracle.pack_range(bs, rows, None, total, w.dst.tables, planes))

    load = dev_plan(w, "dst", K.KVL_SCATTER, unit_bytes=4096)
    out = dev_plan(w, "dst", K.KVL_GATHER | K.KVL_TOKENS_ALL, unit_bytes=4096)
    assert out.payload_bytes == n_out
    host = [torch.zeros(n, dtype=torch.uint8, pin_memory=True) for _ in range(H)]
    out_host = [torch.zeros(n_out, dtype=torch.uint8, pin_memory=True) for _ in range(Ho)]
    slots = [planes_to_dev(W.sentinel_pool(w, "dst", 0xEE)) for _ in range(S)]
    staging = torch.zeros(3 * 8192, dtype=torch.uint8, device="cuda")
    out_staging = torch.zeros(2 * 8192, dtype=torch.uint8, device="cuda") if out_chunk else None
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    got_out, drained = [], []

    def fill(layer, slot):
        host[slot].numpy()[:] = payloads[layer]

    def compute(layer, slot, stream_handle):
        with torch.cuda.stream(ms):
            for pl in slots[slot]:
                pl.add_(1)

    def drain(layer, slot):
        drained.append((layer, slot))
        got_out.append(out_host[slot].numpy().copy())

    torch.cuda.synchronize()
    st = K.kvl_stream_layers(load, host, slots, staging if in_chunk else None, in_chunk, 0, cs, ks, ms, n_layers=L,
                             host_fill=fill, compute=compute, out_plan=out, out_host_layers=out_host,
                             out_staging=out_staging, out_chunk_bytes=out_chunk, host_drain=drain,
                             per_layer_times=True)
    assert drained == [(l, l % Ho) for l in range(L)]
    for l in range(L):
        assert same_bytes(got_out[l], want_out[l]), f"layer {l}: what left for host memory differs from the oracle"
    assert st["d2h_bytes"] == n_out * L and st["h2d_bytes"] == n * L
    # a layer leaves after its compute, and its slot is loaded again only after it has left
    assert np.all(st["t_out_done"] >= st["t_compute_end"] - 1e-3)
    assert np.all(st["t_loaded"][S:] >= st["t_out_done"][:-S] - 1e-3)
    # an outflow plan over another pool geometry is refused
    other = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks + 1), w.hit, w.app, w.dst.tables,
                       K.KVL_GATHER | K.KVL_TOKENS_ALL)
    with pytest.raises(K.KvlError) as e:
        K.kvl_stream_layers(load, host, slots, staging, 8192, 0, cs, ks, ms, n_layers=L, out_plan=other,
                            out_host_layers=out_host, out_staging=out_staging, out_chunk_bytes=out_chunk)
    assert e.value.code == K.KVL_EINVAL


@pytest.mark.parametrize("name,make", [c for c in CASES if c[0] in ("tiny-random", "tiny-3planes", "cfg1", "cfg2-small",
                                                                      "cfg4-small", "token-granular")],
                         ids=lambda v: v if isinstance(v, str) else "")
@pytest.mark.parametrize("groups", [1, 3, 64])
def test_few_workgroups_walking_over_the_tiles(name, make, groups):
    """max_groups: the tiled kernels with fewer workgroups than tiles, each walking over several."""
    w = make()
    run_hop(w, max_groups=groups)
    run_hop(w, max_groups=groups, variant=1 + (3 | 4 | 8), block_threads=128)          # two vectors per lane
    run_range_hop(w, K.KVL_TOKENS_ALL, max_groups=groups, unit_bytes=3000)


def test_pinned_buffers_take_the_thin_kernels_by_default():
    """A transfer buffer or Full-Block buffer in pinned host memory: the kernels that cross the
    host link run with at most 64 workgroups (more tiles than that here), and say the same."""
    w = W.config(3, n_requests=12, token_scale=1 / 16)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool(w, 0, "src")
    want_x = oracle.pack(bs, rows, w.hit, w.src.tables, src)
    g = dev_plan(w, "src", K.KVL_GATHER)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    assert g.payload_bytes > 64 * 8192 * 4                       # far more tiles than workgroups
    host = torch.zeros(g.payload_bytes, dtype=torch.uint8).pin_memory()
    d_src = planes_to_dev(src)
    torch.cuda.synchronize()
    K.kvl_pack_layer(g, d_src, host)
    torch.cuda.synchronize()
    assert same_bytes(host.numpy(), want_x)
    want = W.sentinel_pool(w, "dst")
    oracle.unpack(bs, rows, w.hit, w.dst.tables, want_x, want)
    for forced in (0, 0xFFFFFFFF):                               # default (thin) and "never walk"
        s.set_tuning(max_groups=forced)
        d_dst = planes_to_dev(W.sentinel_pool(w, "dst"))
        K.kvl_unpack_layer(s, host, d_dst)
        torch.cuda.synchronize()
        for a, b in zip(d_dst, want):
            assert same_bytes(to_host(a), b)
