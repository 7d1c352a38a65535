"""Full-size parity: the configurations of the benchmark, in the launch
configuration the benchmark times (default tuning), against the CPU oracle.

Configs 2-4: one layer each, every byte of the transfer buffer and of the
destination pool compared with the oracle's.  Config 5: all 61 layers streamed
from pinned host memory; the oracle computes the first 16 bytes of every token
row of every layer (a 16-byte-row instance of the same definition), which names
the layer and the row and so pins both placement and layer ordering; the device
path is compared on probes taken by each layer's compute kernel and on all rows
of the slots left at the end.
"""
import time

import numpy as np
import pytest
import torch

import kvl_workloads as W
import oracle
import paper_2602_21548_amd as K
from gpu_util import dev_plan, same_bytes, to_host

pytestmark = pytest.mark.gpu

THREADS = 16


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_full_size_layer(idx):
    t0 = time.perf_counter()
    w = W.config(idx)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    layer = idx                                   # any layer: each has its own pool contents
    src = W.fill_pool_fast(w, layer, "src")
    want_x = oracle.pack(bs, rows, w.hit, w.src.tables, src, threads=THREADS)
    g = dev_plan(w, "src", K.KVL_GATHER)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    n = g.payload_bytes
    assert n == want_x.size
    d_src = [torch.from_numpy(p).cuda() for p in src]
    guard = 1 << 16
    d_x = torch.full((n + guard,), 0x3C, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, d_src, d_x)
    d_dst = [torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device="cuda") for r in rows]
    K.kvl_unpack_layer(s, d_x, d_dst)
    torch.cuda.synchronize()
    print(f"[cfg{idx}] inputs + oracle pack + gpu: {time.perf_counter() - t0:.1f} s", flush=True)
    got = to_host(d_x)
    assert np.array_equal(got[:n], want_x), "pack differs from the oracle"
    assert np.all(got[n:] == 0x3C), "pack wrote past the payload"
    del got, d_x, d_src
    for p, r in enumerate(rows):
        # the oracle, one plane at a time (planes are independent problems laid out back to back)
        T = g.hit_tokens
        base = sum(T * q for q in rows[:p])
        want = np.full(w.dst.pool_blocks * bs * r, 0xA5, dtype=np.uint8)
        oracle.unpack(bs, (r,), w.hit, w.dst.tables, want_x[base:base + T * r], [want], threads=THREADS)
        assert np.array_equal(to_host(d_dst[p]), want), f"unpack differs from the oracle in plane {p}"
        del want
    print(f"[cfg{idx}] done after {time.perf_counter() - t0:.1f} s", flush=True)
    g.destroy()
    s.destroy()


@pytest.mark.parametrize("idx,flag", [(2, "append"), (3, "all"), (4, "append")])
def test_full_size_token_ranges(idx, flag):
    """The hop after a layer's compute at full size: the appended tail (a few hundred tokens
    per request: the launch-bound regime) or the whole prompt, prefill pool -> decode pool."""
    t0 = time.perf_counter()
    w = W.config(idx)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    kflag = K.KVL_TOKENS_APPEND if flag == "append" else K.KVL_TOKENS_ALL
    zero = np.zeros_like(w.hit)
    first, count = (w.hit, w.app) if flag == "append" else (zero, w.hit + w.app)
    pe = W.fill_pool_fast(w, 1, "dst")
    de = W.fill_pool_fast(w, 2, "src")
    want_x = oracle.pack_range(bs, rows, first, count, w.dst.tables, pe, threads=THREADS)
    g = K.kvl_plan(K.make_layout(w.layout.n_layers, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                   K.KVL_GATHER | kflag)
    s = K.kvl_plan(K.make_layout(w.layout.n_layers, bs, rows, w.src.pool_blocks), w.hit, w.app, w.src.tables,
                   K.KVL_SCATTER | kflag)
    n = g.payload_bytes
    assert n == want_x.size
    d_pe = [torch.from_numpy(p).cuda() for p in pe]
    d_de = [torch.from_numpy(p).cuda() for p in de]
    d_x = torch.full((n + 4096,), 0x3C, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, d_pe, d_x)
    K.kvl_unpack_layer(s, d_x, d_de)
    torch.cuda.synchronize()
    got = to_host(d_x)
    assert np.array_equal(got[:n], want_x) and np.all(got[n:] == 0x3C)
    oracle.unpack_range(bs, rows, first, count, w.src.tables, want_x, de, threads=THREADS)   # de becomes the expectation
    for p in range(len(rows)):
        assert np.array_equal(to_host(d_de[p]), de[p]), f"merged decode-side pool differs in plane {p}"
    print(f"[cfg{idx} {flag}] {n / 1e6:.1f} MB payload, done after {time.perf_counter() - t0:.1f} s", flush=True)
    g.destroy()
    s.destroy()


def test_full_size_full_blocks_from_pinned_host():
    """Storage layout at its real shape: 61-layer Full Blocks of 64 x 1152 bytes per layer in
    pinned host memory; every layer loaded into the paged pool by one kernel reading the host
    buffer, compared with the oracle on two layers in full and on the row heads of all layers."""
    t0 = time.perf_counter()
    w = W.config(3, n_requests=3)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    row = rows[0]
    s = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                   K.KVL_SCATTER | K.KVL_NO_MERGE)
    fb, nfb = s.fullblock_geometry()
    assert fb == L * bs * row
    host = torch.empty(fb * nfb, dtype=torch.uint8, pin_memory=True)
    a = host.numpy()
    rng = np.random.Generator(np.random.PCG64(W.BASE_SEED + 405))
    tile = rng.integers(0, 256, size=1 << 24, dtype=np.uint8)
    for pos in range(0, a.size, tile.size):
        k = min(tile.size, a.size - pos)
        a[pos:pos + k] = tile[:k]
    # head of every row of every block and layer: (block, layer, row) -- names where it must land
    heads = a.reshape(nfb, L, bs, row)[:, :, :, :8].view(np.uint64).reshape(nfb, L, bs)
    heads[:] = (np.arange(nfb, dtype=np.uint64)[:, None, None] << np.uint64(32)) \
        | (np.arange(L, dtype=np.uint64)[None, :, None] << np.uint64(16)) | np.arange(bs, dtype=np.uint64)[None, None, :]
    print(f"[fullblocks] {nfb} Full Blocks x {fb} B = {a.size / 1e9:.2f} GB pinned after {time.perf_counter() - t0:.1f} s", flush=True)
    pool = [torch.full((w.dst.pool_blocks * bs * row,), 0xA5, dtype=torch.uint8, device="cuda")]
    st = torch.cuda.Stream()
    zero = np.zeros_like(w.hit)
    # 8-byte-row instance of the same definition for the row heads of every layer
    head_buf = np.ascontiguousarray(a.reshape(nfb, L, bs, row)[:, :, :, :8]).reshape(-1)
    chunk = 32 << 20
    staging = torch.empty(2 * chunk, dtype=torch.uint8, device="cuda")
    cs = torch.cuda.Stream()
    for l in range(L):
        torch.cuda.synchronize()
        if l % 2:       # odd layers by the staged form: strided copies into HBM slots, converting kernels there
            K.kvl_h2d_fullblocks_layer(s, host, l, staging, chunk, pool, cs, st)
        else:           # even layers by the one kernel that reads the host buffer itself
            K.kvl_fullblocks_to_pool_layer(s, host, l, pool, stream=st)
        st.synchronize()
        cs.synchronize()
        want_h = [np.full(w.dst.pool_blocks * bs * 8, 0xA5, dtype=np.uint8)]
        oracle.fullblocks_to_pool(bs, L, (8,), zero, w.hit, w.dst.tables, l, head_buf, want_h)
        got_h = pool[0].view(-1, row)[:, :8].contiguous()
        assert same_bytes(to_host(got_h).reshape(-1), want_h[0]), f"layer {l}: rows landed in the wrong place"
        if l in (0, L - 1):
            want = [np.full(w.dst.pool_blocks * bs * row, 0xA5, dtype=np.uint8)]
            oracle.fullblocks_to_pool(bs, L, rows, zero, w.hit, w.dst.tables, l, a, want)
            assert np.array_equal(to_host(pool[0]), want[0]), f"layer {l} differs from the oracle"
    # and back: the pool of the last layer persisted into a fresh buffer's layer 5 by the staged form
    g = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                   K.KVL_GATHER | K.KVL_NO_MERGE)
    last = [to_host(pool[0])]
    want_back = a.copy()
    oracle.pool_to_fullblocks(bs, L, rows, zero, w.hit, w.dst.tables, 5, last, want_back)
    K.kvl_d2h_fullblocks_layer(g, pool, 5, staging, chunk, host, st, cs)
    st.synchronize()
    cs.synchronize()
    assert np.array_equal(a, want_back), "staged persist differs from the oracle"
    print(f"[fullblocks] done after {time.perf_counter() - t0:.1f} s", flush=True)
    s.destroy()
    g.destroy()


@pytest.mark.parametrize("idx", [2, 4])
def test_full_size_fused_move(idx):
    t0 = time.perf_counter()
    w = W.config(idx)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool_fast(w, 7, "src")
    x = oracle.pack(bs, rows, w.hit, w.src.tables, src, threads=THREADS)
    g = dev_plan(w, "src", K.KVL_GATHER)
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    m = K.kvl_plan_pair(g, s)
    d_src = [torch.from_numpy(p).cuda() for p in src]
    d_dst = [torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device="cuda") for r in rows]
    K.kvl_move_layer(m, d_src, d_dst)
    torch.cuda.synchronize()
    T = g.hit_tokens
    for p, r in enumerate(rows):
        base = sum(T * q for q in rows[:p])
        want = np.full(w.dst.pool_blocks * bs * r, 0xA5, dtype=np.uint8)
        oracle.unpack(bs, (r,), w.hit, w.dst.tables, x[base:base + T * r], [want], threads=THREADS)
        assert np.array_equal(to_host(d_dst[p]), want), f"plane {p}"
    print(f"[cfg{idx} move] done after {time.perf_counter() - t0:.1f} s", flush=True)


def test_full_size_streamed_layers():
    t0 = time.perf_counter()
    w = W.config(5)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    row = rows[0]
    H, S = w.notes["host_slots"], w.notes["dev_slots"]
    s = dev_plan(w, "dst", K.KVL_SCATTER)
    n, T = s.payload_bytes, s.hit_tokens
    pool_rows = w.dst.pool_blocks * bs

    # host buffers: a random tile repeated; the first 16 bytes of row g of layer l are (l, g)
    rng = np.random.Generator(np.random.PCG64(W.BASE_SEED + 205))
    tile = rng.integers(0, 256, size=1 << 24, dtype=np.uint8)
    host = [torch.empty(n, dtype=torch.uint8, pin_memory=True) for _ in range(H)]
    for h in host:
        a = h.numpy()
        for pos in range(0, n, tile.size):
            k = min(tile.size, n - pos)
            a[pos:pos + k] = tile[:k]
    g_idx = np.arange(T, dtype=np.uint64)

    def tags_of(layer):
        t = np.empty((T, 2), dtype=np.uint64)
        t[:, 0] = layer
        t[:, 1] = g_idx
        return t

    def fill(layer, slot):
        host[slot].numpy().reshape(T, row)[:, :16] = tags_of(layer).view(np.uint8).reshape(T, 16)

    # oracle on 16-byte rows: what the head of every pool row must be when layer l is computed
    o_slots = [[np.full(pool_rows * 16, 0xA5, dtype=np.uint8)] for _ in range(S)]
    o_host = [np.zeros(T * 16, dtype=np.uint8) for _ in range(H)]
    rs = np.random.Generator(np.random.PCG64(W.BASE_SEED + 305))
    probe_rows = np.sort(rs.choice(pool_rows, size=512, replace=False))
    probes = [(0, int(r) * row) for r in probe_rows]
    want_probe = np.zeros((L, len(probes), 16), dtype=np.uint8)
    gen = oracle.stream_layers(bs, (16,), w.hit, w.dst.tables, o_host, L, o_slots)
    want_final = {}
    for l in range(L):
        o_host[l % H][:] = tags_of(l).view(np.uint8).reshape(-1)
        _, sl, planes = next(gen)
        want_probe[l] = planes[0].reshape(pool_rows, 16)[probe_rows]
        if l >= L - S:
            want_final[sl] = planes[0].copy()
    print(f"[cfg5] oracle done after {time.perf_counter() - t0:.1f} s", flush=True)

    slots = [[torch.full((pool_rows * row,), 0xA5, dtype=torch.uint8, device="cuda")] for _ in range(S)]
    chunk = 128 << 20
    staging = torch.empty(4 * chunk, dtype=torch.uint8, device="cuda")
    probe_out = torch.zeros(L * len(probes) * 16, dtype=torch.uint8, device="cuda")
    # two layers from the middle of the run are kept whole, every byte of the slot as their compute saw it
    whole_layers = [L // 3, (2 * L) // 3 + 1]
    snaps = [[torch.empty(pool_rows * row, dtype=torch.uint8, device="cuda")] if l in whole_layers else None
             for l in range(L)]
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    st = K.kvl_stream_layers(s, host, slots, staging, chunk, w.notes["compute_us"], cs, ks, ms,
                             probes=probes, probe_out=probe_out, host_fill=fill, per_layer_times=True,
                             snapshots=snaps)
    print(f"[cfg5] streamed {L} layers in {st['total_ms']:.0f} ms ({st['link_gbps']:.1f} GB/s) "
          f"after {time.perf_counter() - t0:.1f} s", flush=True)
    got = to_host(probe_out).reshape(L, len(probes), 16)
    for l in range(L):
        assert got[l].tobytes() == want_probe[l].tobytes(), f"compute of layer {l} saw the wrong cache"
    for sl, want in want_final.items():
        head = slots[sl][0].view(pool_rows, row)[:, :16].contiguous()
        assert same_bytes(to_host(head).reshape(-1), want), f"slot {sl} differs from the oracle at the end"
    # beyond the 16-byte heads: the rest of every hit row is the host buffer's bytes, and rows
    # without a hit token still hold the sentinel -- checked on a sample of whole rows
    last_slot = (L - 1) % S
    pool = slots[last_slot][0].view(pool_rows, row)
    hb = host[(L - 1) % H].numpy().reshape(T, row)
    heads = want_final[last_slot].reshape(pool_rows, 16)
    for r in probe_rows[:128]:
        got_row = to_host(pool[int(r)])
        if np.all(heads[r] == 0xA5):
            assert np.all(got_row == 0xA5)
        else:
            gi = int(heads[r].view(np.uint64)[1])
            assert got_row.tobytes() == hb[gi].tobytes()
    tl, tb, te = st["t_loaded"], st["t_compute_begin"], st["t_compute_end"]
    assert np.all(tb >= tl - 1e-3) and np.all(te - tb >= 0.18) and np.all(np.diff(tb) > 0)
    # load of layer l + S does not finish before compute of layer l has ended
    assert np.all(tl[S:] >= te[:-S] - 1e-3)
    # The whole slot of two middle layers.  The oracle, run once more on 16-byte rows, says which
    # host row (layer, g) every pool row must hold; the bytes after a row's head are the host
    # buffer's, which is the repeated tile whatever the layer.  Rows are compared in slices.
    gen = oracle.stream_layers(bs, (16,), w.hit, w.dst.tables, o_host, max(whole_layers) + 1,
                               [[np.full(pool_rows * 16, 0xA5, dtype=np.uint8)] for _ in range(S)])
    for l in range(max(whole_layers) + 1):
        o_host[l % H][:] = tags_of(l).view(np.uint8).reshape(-1)
        _, _, planes = next(gen)
        if l not in whole_layers:
            continue
        heads = planes[0].reshape(pool_rows, 16)
        got = to_host(snaps[l][0]).reshape(pool_rows, row)
        assert same_bytes(np.ascontiguousarray(got[:, :16]).reshape(-1), planes[0]), f"layer {l}: row heads"
        empty = np.all(heads == 0xA5, axis=1)
        assert np.all(heads[~empty].view(np.uint64).reshape(-1, 2)[:, 0] == l)
        gi = heads.view(np.uint64).reshape(pool_rows, 2)[:, 1]
        step = 1 << 18
        for lo in range(0, pool_rows, step):
            hi = min(pool_rows, lo + step)
            e = empty[lo:hi]
            blk = got[lo:hi]
            assert np.all(blk[e] == 0xA5), f"layer {l}: a row without a hit token was written"
            pos = gi[lo:hi][~e].astype(np.int64)[:, None] * row + np.arange(16, row, dtype=np.int64)[None, :]
            assert np.array_equal(blk[~e][:, 16:], tile[pos % tile.size]), f"layer {l}: rows {lo}..{hi}"
    print(f"[cfg5] layers {whole_layers} compared whole after {time.perf_counter() - t0:.1f} s", flush=True)
    s.destroy()


def test_row_indices_at_the_32_bit_limit():
    """The largest pool a plan accepts: block_tokens * pool_blocks just below 2^32 token rows
    (descriptors index rows with 32 bits), 68.7 GB per pool at 16-byte rows.  A few requests
    use the first block, the last blocks and blocks in between.  The oracle works on the same
    problem with the touched blocks renumbered 0, 1, 2, ... (a pool of only those blocks):
    the bytes it expects in the transfer buffer and in every touched block are the same."""
    bs, row = 64, 16
    pool_blocks = (2 ** 32 - 1) // bs                     # one more block and kvl_plan says KVL_ERANGE
    blk = bs * row
    rng = np.random.Generator(np.random.PCG64(W.BASE_SEED + 977))
    hit = np.array([100, 64, 130, 1], dtype=np.uint32)
    app = np.array([0, 5, 0, 0], dtype=np.uint32)
    mid = pool_blocks // 2
    src_ids = [[pool_blocks - 1, 0], [pool_blocks - 2, 12345678], [mid, mid + 1, 3], [pool_blocks - 3]]
    dst_ids = [[7, pool_blocks - 1], [mid - 1, 1], [pool_blocks - 4, pool_blocks - 3, pool_blocks - 2], [0]]
    with pytest.raises(K.KvlError) as e:
        K.kvl_plan(K.make_layout(1, bs, (row,), pool_blocks + 1), hit, app,
                   [np.array(t, np.int32) for t in src_ids], K.KVL_GATHER | K.KVL_HOST_ONLY)
    assert e.value.code == K.KVL_ERANGE

    def compact(ids):
        order = sorted({b for t in ids for b in t})
        number = {b: i for i, b in enumerate(order)}
        return order, [np.array([number[b] for b in t], np.int32) for t in ids]

    src_order, src_small = compact(src_ids)
    dst_order, dst_small = compact(dst_ids)
    small_src = rng.integers(0, 256, size=len(src_order) * blk, dtype=np.uint8)
    want_x = oracle.pack(bs, (row,), hit, src_small, [small_src])
    small_dst = np.full(len(dst_order) * blk, 0xA5, dtype=np.uint8)
    oracle.unpack(bs, (row,), hit, dst_small, want_x, [small_dst])

    torch.cuda.empty_cache()
    lay = K.make_layout(1, bs, (row,), pool_blocks)
    g = K.kvl_plan(lay, hit, app, [np.array(t, np.int32) for t in src_ids], K.KVL_GATHER)
    s = K.kvl_plan(lay, hit, app, [np.array(t, np.int32) for t in dst_ids], K.KVL_SCATTER)
    d_src = torch.empty(pool_blocks * blk, dtype=torch.uint8, device="cuda")      # only touched blocks are set
    d_dst = torch.empty(pool_blocks * blk, dtype=torch.uint8, device="cuda")
    for i, b in enumerate(src_order):
        d_src[b * blk:(b + 1) * blk] = torch.from_numpy(small_src[i * blk:(i + 1) * blk]).cuda()
    for b in dst_order:
        d_dst[b * blk:(b + 1) * blk] = 0xA5
    n = g.payload_bytes
    d_x = torch.full((n + 4096,), 0x3C, dtype=torch.uint8, device="cuda")
    K.kvl_pack_layer(g, [d_src], d_x)
    K.kvl_unpack_layer(s, d_x, [d_dst])
    torch.cuda.synchronize()
    got = to_host(d_x)
    assert same_bytes(got[:n], want_x) and np.all(got[n:] == 0x3C)
    for i, b in enumerate(dst_order):
        assert same_bytes(to_host(d_dst[b * blk:(b + 1) * blk]), small_dst[i * blk:(i + 1) * blk]), f"block {b}"
    # the fused move between the two pools gives the same destination blocks
    for b in dst_order:
        d_dst[b * blk:(b + 1) * blk] = 0xA5
    m = K.kvl_plan_pair(g, s)
    K.kvl_move_layer(m, [d_src], [d_dst])
    torch.cuda.synchronize()
    for i, b in enumerate(dst_order):
        assert same_bytes(to_host(d_dst[b * blk:(b + 1) * blk]), small_dst[i * blk:(i + 1) * blk]), f"move: block {b}"
    for p in (m, g, s):
        p.destroy()
    del d_src, d_dst, d_x
    torch.cuda.empty_cache()


def test_full_size_streamed_layers_with_outflow():
    """Six layers of the streamed workload at full size, with every computed layer (hit and
    appended rows) leaving for pinned host memory while the next ones are loaded.  The oracle
    works on the first 16 bytes of every row, as above; whole rows are checked on a sample."""
    t0 = time.perf_counter()
    w = W.config(5)
    L, bs, rows = 6, w.layout.block_tokens, w.layout.row_bytes
    row = rows[0]
    H = S = Ho = 2
    lay = K.make_layout(w.layout.n_layers, bs, rows, w.dst.pool_blocks)
    s = K.kvl_plan(lay, w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
    out = K.kvl_plan(lay, w.hit, w.app, w.dst.tables, K.KVL_GATHER | K.KVL_TOKENS_ALL)
    n, T = s.payload_bytes, s.hit_tokens
    total = (w.hit + w.app).astype(np.uint32)
    T_all = int(total.astype(np.int64).sum())
    assert out.payload_bytes == T_all * row
    pool_rows = w.dst.pool_blocks * bs
    rng = np.random.Generator(np.random.PCG64(W.BASE_SEED + 206))
    tile = rng.integers(0, 256, size=1 << 24, dtype=np.uint8)
    host = [torch.empty(n, dtype=torch.uint8, pin_memory=True) for _ in range(H)]
    for h in host:
        a = h.numpy()
        for pos in range(0, n, tile.size):
            k = min(tile.size, n - pos)
            a[pos:pos + k] = tile[:k]
    out_host = [torch.zeros(T_all * row, dtype=torch.uint8, pin_memory=True) for _ in range(Ho)]
    g_idx = np.arange(T, dtype=np.uint64)

    def tags_of(layer):
        t = np.empty((T, 2), dtype=np.uint64)
        t[:, 0] = layer
        t[:, 1] = g_idx
        return t

    def fill(layer, slot):
        host[slot].numpy().reshape(T, row)[:, :16] = tags_of(layer).view(np.uint8).reshape(T, 16)

    o_slots = [[np.full(pool_rows * 16, 0xA5, dtype=np.uint8)] for _ in range(S)]
    o_host = [np.zeros(T * 16, dtype=np.uint8) for _ in range(H)]
    want_heads = []
    gen = oracle.stream_layers(bs, (16,), w.hit, w.dst.tables, o_host, L, o_slots)
    for l in range(L):
        o_host[l % H][:] = tags_of(l).view(np.uint8).reshape(-1)
        _, _, planes = next(gen)
        want_heads.append(oracle.pack_range(bs, (16,), None, total, w.dst.tables, planes, threads=THREADS))
    print(f"[cfg5 outflow] oracle done after {time.perf_counter() - t0:.1f} s", flush=True)

    slots = [[torch.full((pool_rows * row,), 0xA5, dtype=torch.uint8, device="cuda")] for _ in range(S)]
    chunk = 128 << 20
    staging = torch.empty(2 * chunk, dtype=torch.uint8, device="cuda")
    out_staging = torch.empty(chunk, dtype=torch.uint8, device="cuda")
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    rs = np.random.Generator(np.random.PCG64(W.BASE_SEED + 306))
    sample = np.sort(rs.choice(T_all, size=256, replace=False))
    # where out-row j comes from: request r, token t; a hit token's row is the host buffer's
    ends = np.cumsum(total.astype(np.int64))
    hit_starts = np.concatenate(([0], np.cumsum(w.hit.astype(np.int64))))
    seen = []

    def drain(layer, slot):
        got = out_host[slot].numpy().reshape(T_all, row)
        heads = np.ascontiguousarray(got[:, :16]).reshape(-1)
        assert same_bytes(heads, want_heads[layer]), f"layer {layer}: outflow heads differ from the oracle"
        for j in sample:
            r = int(np.searchsorted(ends, j, side="right"))
            t = int(j - (ends[r] - total[r]))
            if t < w.hit[r]:
                assert got[j, 16:].tobytes() == tile_row(int(hit_starts[r]) + t), f"layer {layer} out-row {j}"
            else:
                assert np.all(got[j] == 0xA5), f"layer {layer} out-row {j}: an appended row nobody wrote"
        seen.append(layer)

    def tile_row(g):
        # bytes 16.. of host row g: the repeated tile, whatever the layer
        pos = g * row + 16
        idx = (pos + np.arange(row - 16)) % tile.size
        return tile[idx].tobytes()

    torch.cuda.synchronize()
    st = K.kvl_stream_layers(s, host, slots, staging, chunk, w.notes["compute_us"], cs, ks, ms, n_layers=L,
                             host_fill=fill, out_plan=out, out_host_layers=out_host, out_staging=out_staging,
                             out_chunk_bytes=chunk, host_drain=drain)
    assert seen == list(range(L))
    print(f"[cfg5 outflow] {L} layers in {st['total_ms']:.0f} ms: in {st['link_gbps']:.1f} GB/s, "
          f"out {st['out_gbps']:.1f} GB/s, after {time.perf_counter() - t0:.1f} s", flush=True)
    s.destroy()
    out.destroy()
