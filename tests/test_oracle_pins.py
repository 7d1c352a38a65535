"""Pins for the CPU oracle: checks against things other than itself.

The paper prints no worked example for the cache-load path, so the oracle is
pinned by what the definition (Appendix A.5 layout, Section 4.1 "hit tokens of
this layer") and plain mathematics fix: an independent per-byte brute force,
library routines it must reduce to (memcpy, numpy.take), algebraic identities,
and a closed-form fill.  A last test plants mistakes in copies of the C source
and demands that the pins notice each of them.
"""
import itertools
import os
import re
import subprocess
import sys
import tempfile

import numpy as np
import pytest

import kvl_workloads as W
import oracle
from oracle import kvl_oracle as KO


# --------------------------------------------------------------------------
# independent brute force (pure Python, different structure from the C loops)
# --------------------------------------------------------------------------

def brute_pack(bs, row_bytes, hit, tables, pools):
    """Walk the *output* byte by byte and ask where it comes from."""
    T = sum(int(h) for h in hit)
    out = bytearray()
    for p, row in enumerate(row_bytes):
        for g in range(T):                 # g-th hit token of the batch
            r, t = 0, g
            while t >= int(hit[r]):        # which request, which token of it
                t -= int(hit[r])
                r += 1
            blk, within = divmod(t, bs)
            start = (int(tables[r][blk]) * bs + within) * row
            out += bytes(pools[p][start:start + row])
    return np.frombuffer(bytes(out), dtype=np.uint8)


def brute_hit_mask(bs, row, hit, tables, pool_blocks):
    """Boolean per pool byte: does a hit token live here?"""
    m = np.zeros(pool_blocks * bs * row, dtype=bool)
    for r, h in enumerate(hit):
        for t in range(int(h)):
            ph = int(tables[r][t // bs]) * bs + (t % bs)
            m[ph * row:(ph + 1) * row] = True
    return m


def brute_unpack(bs, row_bytes, hit, tables, xfer, pools):
    T = sum(int(h) for h in hit)
    pos = 0
    for p, row in enumerate(row_bytes):
        for r, h in enumerate(hit):
            for t in range(int(h)):
                ph = int(tables[r][t // bs]) * bs + (t % bs)
                pools[p][ph * row:(ph + 1) * row] = xfer[pos:pos + row]
                pos += row
    assert pos == T * sum(row_bytes)


def _o_pack(w, pools, side="src", **kw):
    s = w.src if side == "src" else w.dst
    return oracle.pack(w.layout.block_tokens, w.layout.row_bytes, w.hit, s.tables, pools, **kw)


def _o_unpack(w, xfer, pools, side="dst", **kw):
    s = w.src if side == "src" else w.dst
    oracle.unpack(w.layout.block_tokens, w.layout.row_bytes, w.hit, s.tables, xfer, pools, **kw)


TINY = [
    dict(seed=1, n_requests=3, block_tokens=1, row_bytes=(16,), pool_blocks=40, max_tokens=9),
    dict(seed=2, n_requests=4, block_tokens=2, row_bytes=(48,), pool_blocks=64, max_tokens=17),
    dict(seed=3, n_requests=5, block_tokens=16, row_bytes=(656,), pool_blocks=32, max_tokens=70),
    dict(seed=4, n_requests=3, block_tokens=16, row_bytes=(32, 16), pool_blocks=24, max_tokens=60),
    dict(seed=5, n_requests=6, block_tokens=4, row_bytes=(16, 48), pool_blocks=64, max_tokens=30, kind="runs"),
    dict(seed=6, n_requests=2, block_tokens=3, row_bytes=(5,), pool_blocks=20, max_tokens=20),  # odd row size
    dict(seed=7, n_requests=4, block_tokens=8, row_bytes=(16,), pool_blocks=30, max_tokens=40, kind="contiguous"),
]


# --------------------------------------------------------------------------
# the pin battery (also used by the planted-mistake test)
# --------------------------------------------------------------------------

def pin_brute_force():
    for kw in TINY:
        w = W.tiny(**kw)
        pools = W.fill_pool(w, 0, "src")
        got = _o_pack(w, pools)
        want = brute_pack(w.layout.block_tokens, w.layout.row_bytes, w.hit, w.src.tables, pools)
        assert got.tobytes() == want.tobytes(), kw
        # unpack of an arbitrary byte string into a sentinel pool
        x = W.random_payload(w, 0, got.size)
        dst = W.sentinel_pool(w, "dst")
        ref = [d.copy() for d in dst]
        _o_unpack(w, x, dst)
        brute_unpack(w.layout.block_tokens, w.layout.row_bytes, w.hit, w.dst.tables, x, ref)
        for a, b in zip(dst, ref):
            assert a.tobytes() == b.tobytes(), kw


def pin_exhaustive_permutations():
    bs, row = 2, 16
    rng = np.random.Generator(np.random.PCG64(99))
    pool = rng.integers(0, 256, size=5 * bs * row, dtype=np.uint8)
    for n in range(1, 6):
        for perm in itertools.permutations(range(5), n):
            hit = [n * bs - 1]  # ragged: last block holds one row
            tables = [np.array(perm, dtype=np.int32)]
            got = oracle.pack(bs, (row,), hit, tables, [pool])
            want = brute_pack(bs, (row,), hit, tables, [pool])
            assert got.tobytes() == want.tobytes(), perm


def pin_round_trip():
    for kw in TINY + [dict(seed=11, n_requests=8, block_tokens=16, row_bytes=(1152,), pool_blocks=200, max_tokens=300)]:
        w = W.tiny(**kw)
        src = W.fill_pool(w, 0, "src")
        x = _o_pack(w, src, "src")
        # same table on the way back: hit rows restored, everything else sentinel
        back = W.sentinel_pool(w, "src", 0xA5)
        _o_unpack(w, x, back, "src")
        for p, row in enumerate(w.layout.row_bytes):
            m = brute_hit_mask(w.layout.block_tokens, row, w.hit, w.src.tables, w.src.pool_blocks)
            assert np.array_equal(back[p][m], src[p][m])
            assert np.all(back[p][~m] == 0xA5)
        # other table: pack(unpack(x)) == x for an arbitrary byte string
        y = W.random_payload(w, 1, x.size)
        dst = W.sentinel_pool(w, "dst")
        _o_unpack(w, y, dst, "dst")
        assert _o_pack(w, dst, "dst").tobytes() == y.tobytes()


def pin_byte_conservation():
    for kw in TINY:
        w = W.tiny(**kw)
        T = int(np.sum(w.hit.astype(np.int64)))
        n = T * sum(w.layout.row_bytes)
        assert oracle.payload_bytes(w.hit, w.layout.row_bytes) == n
        assert oracle.total_hit_tokens(w.hit) == T
        guard = 64
        buf = np.full(n + guard, 0x5C, dtype=np.uint8)
        src = [np.where(p == 0x5C, np.uint8(0x5D), p) for p in W.fill_pool(w, 0, "src")]  # never 0x5C
        _o_pack(w, src, xfer=buf)
        assert np.all(buf[n:] == 0x5C)            # guard untouched
        assert np.all(buf[:n] != 0x5C)            # every payload byte written
        dst = W.sentinel_pool(w, "dst", 0x5C)
        _o_unpack(w, buf, dst)
        changed = sum(int(np.count_nonzero(d != 0x5C)) for d in dst)
        assert changed == n                       # exactly payload bytes written


def pin_memcpy_and_take():
    rng = np.random.Generator(np.random.PCG64(5))
    bs, row, nblk = 16, 48, 12
    pool = rng.integers(0, 256, size=nblk * bs * row, dtype=np.uint8)
    # identity table, whole blocks: pack is a memcpy of the prefix
    hit = [7 * bs]
    x = oracle.pack(bs, (row,), hit, [np.arange(nblk, dtype=np.int32)], [pool])
    assert x.tobytes() == pool[:7 * bs * row].tobytes()
    # block size 1: pack is a row gather
    tb = [rng.permutation(nblk * bs)[:50].astype(np.int32), rng.permutation(nblk * bs)[:31].astype(np.int32)]
    x = oracle.pack(1, (row,), [50, 31], tb, [pool])
    want = np.take(pool.reshape(-1, row), np.concatenate(tb), axis=0)
    assert x.tobytes() == want.tobytes()
    # and unpack with block size 1 is a row scatter
    dst = np.zeros_like(pool)
    oracle.unpack(1, (row,), [50, 31], tb, x, [dst])
    ref = np.zeros_like(pool).reshape(-1, row)
    ref[np.concatenate(tb)] = want
    assert dst.tobytes() == ref.tobytes()
    # two planes are two independent one-plane problems laid out one after the other
    pool2 = rng.integers(0, 256, size=nblk * bs * 16, dtype=np.uint8)
    hit2 = [37, 5]
    tabs = [np.array([3, 9, 1], np.int32), np.array([0], np.int32)]
    both = oracle.pack(bs, (row, 16), hit2, tabs, [pool, pool2])
    a = oracle.pack(bs, (row,), hit2, tabs, [pool])
    b = oracle.pack(bs, (16,), hit2, tabs, [pool2])
    assert both.tobytes() == a.tobytes() + b.tobytes()


def pin_permutation_algebra():
    rng = np.random.Generator(np.random.PCG64(17))
    bs, row, n = 4, 32, 24
    src = rng.integers(0, 256, size=n * bs * row, dtype=np.uint8)
    pi = rng.permutation(n).astype(np.int32)
    sigma = rng.permutation(n).astype(np.int32)
    hit = [n * bs]
    x = oracle.pack(bs, (row,), hit, [pi], [src])
    dst = np.zeros_like(src)
    oracle.unpack(bs, (row,), hit, [sigma], x, [dst])
    S = src.reshape(n, bs * row)
    D = dst.reshape(n, bs * row)
    for i in range(n):
        assert np.array_equal(D[sigma[i]], S[pi[i]])
    # composing with the inverse hop is the identity
    y = oracle.pack(bs, (row,), hit, [sigma], [dst])
    back = np.zeros_like(src)
    oracle.unpack(bs, (row,), hit, [pi], y, [back])
    assert back.tobytes() == src.tobytes()


def pin_closed_form_fill():
    # every pool byte is a function of (block, row in block, byte); the packed
    # buffer must then be that function of the table entries
    w = W.tiny(seed=21, n_requests=5, block_tokens=16, row_bytes=(80,), pool_blocks=64, max_tokens=100)
    bs, row = 16, 80
    nb = w.src.pool_blocks

    def f(b, t, j):
        v = (b.astype(np.uint64) * np.uint64(2654435761) + t.astype(np.uint64) * np.uint64(40503)
             + j.astype(np.uint64) * np.uint64(97))
        return ((v >> np.uint64(7)) & np.uint64(0xFF)).astype(np.uint8)

    B, Tt, J = np.meshgrid(np.arange(nb), np.arange(bs), np.arange(row), indexing="ij")
    pool = f(B, Tt, J).reshape(-1)
    x = _o_pack(w, [pool])
    pos = 0
    for r, h in enumerate(w.hit):
        t = np.arange(int(h))
        b = w.src.tables[r][t // bs]
        tt, jj = np.meshgrid(t % bs, np.arange(row), indexing="ij")
        bb = np.repeat(b[:, None], row, axis=1)
        want = f(bb, tt, jj).reshape(-1)
        assert x[pos:pos + want.size].tobytes() == want.tobytes()
        pos += want.size
    assert pos == x.size


def pin_threads_agree():
    w = W.tiny(seed=31, n_requests=9, block_tokens=16, row_bytes=(64, 32), pool_blocks=128, max_tokens=150)
    src = W.fill_pool(w, 0, "src")
    a = _o_pack(w, src)
    b = _o_pack(w, src, threads=4)
    assert a.tobytes() == b.tobytes()
    d1, d4 = W.sentinel_pool(w), W.sentinel_pool(w)
    _o_unpack(w, a, d1)
    _o_unpack(w, a, d4, threads=4)
    for u, v in zip(d1, d4):
        assert u.tobytes() == v.tobytes()


def brute_pack_range(bs, row_bytes, first, count, tables, pools):
    out = bytearray()
    for p, row in enumerate(row_bytes):
        for r in range(len(count)):
            for t in range(int(first[r]), int(first[r]) + int(count[r])):
                blk, within = divmod(t, bs)
                start = (int(tables[r][blk]) * bs + within) * row
                out += bytes(pools[p][start:start + row])
    return np.frombuffer(bytes(out), dtype=np.uint8)


def pin_ranges():
    """Token ranges (the appended tail, the whole prompt): brute force, reduction to the
    prefix case, and the merge property of Section 4.1 (hit cache + miss cache = prompt cache)."""
    for kw in TINY:
        w = W.tiny(**kw)
        bs, rows = w.layout.block_tokens, w.layout.row_bytes
        src = W.fill_pool(w, 0, "src")
        zero = np.zeros_like(w.hit)
        # reduction: first = 0, count = hit is the prefix definition
        assert oracle.pack_range(bs, rows, zero, w.hit, w.src.tables, src).tobytes() == _o_pack(w, src).tobytes()
        assert oracle.pack_range(bs, rows, None, w.hit, w.src.tables, src).tobytes() == _o_pack(w, src).tobytes()
        # brute force on the tail and on an arbitrary inner range
        tail = oracle.pack_range(bs, rows, w.hit, w.app, w.src.tables, src)
        assert tail.tobytes() == brute_pack_range(bs, rows, w.hit, w.app, w.src.tables, src).tobytes(), kw
        tot = w.hit + w.app
        f2 = tot // 3
        c2 = tot - f2 - tot // 4
        inner = oracle.pack_range(bs, rows, f2, c2, w.src.tables, src)
        assert inner.tobytes() == brute_pack_range(bs, rows, f2, c2, w.src.tables, src).tobytes(), kw
        # merge: scattering the hit part and then the tail equals scattering the whole prompt
        whole = oracle.pack_range(bs, rows, zero, tot, w.src.tables, src)
        hitp = _o_pack(w, src)
        a = W.sentinel_pool(w, "dst")
        b = W.sentinel_pool(w, "dst")
        oracle.unpack_range(bs, rows, zero, tot, w.dst.tables, whole, a)
        oracle.unpack(bs, rows, w.hit, w.dst.tables, hitp, b)
        oracle.unpack_range(bs, rows, w.hit, w.app, w.dst.tables, tail, b)
        for u, v in zip(a, b):
            assert u.tobytes() == v.tobytes(), kw
        # the whole-prompt buffer is, per plane and request, the hit rows followed by the tail rows
        T_h, T_a, T_w = int(w.hit.sum()), int(w.app.sum()), int(tot.sum())
        ph = pa = pw = 0
        for p, row in enumerate(rows):
            ph, pa, pw = sum(T_h * q for q in rows[:p]), sum(T_a * q for q in rows[:p]), sum(T_w * q for q in rows[:p])
            for r in range(len(tot)):
                nh, na = int(w.hit[r]) * row, int(w.app[r]) * row
                assert whole[pw:pw + nh].tobytes() == hitp[ph:ph + nh].tobytes()
                assert whole[pw + nh:pw + nh + na].tobytes() == tail[pa:pa + na].tobytes()
                ph, pa, pw = ph + nh, pa + na, pw + nh + na
        # threads agree
        assert oracle.pack_range(bs, rows, w.hit, w.app, w.src.tables, src, threads=3).tobytes() == tail.tobytes()
    # range scatter preconditions: a shared boundary block between two requests' ranges is an alias
    tabs = [np.array([1, 2], np.int32), np.array([2, 3], np.int32)]
    assert oracle.check_range_scatter(4, 8, [0, 0], [5, 3], tabs) == oracle.E_DUP    # both touch block 2
    assert oracle.check_range_scatter(4, 8, [0, 0], [4, 3], tabs) == oracle.OK      # first stops inside block 1
    assert oracle.check_range_scatter(4, 8, [0, 4], [5, 3], tabs) == oracle.OK      # second starts in block 3
    assert oracle.check_range_scatter(4, 8, [0, 0], [0, 0], tabs) == oracle.OK
    assert oracle.check_range_scatter(4, 3, [0, 4], [4, 3], tabs) == oracle.E_BLOCK


def pin_full_blocks():
    """Storage layout (Appendix A.5): a Full Block is the concatenation of a block's Layer
    Blocks.  Checked against NumPy reshapes of that sentence, a per-byte brute force, the
    Layer-Block path, and a store/load round trip."""
    # (1) one plane, whole blocks: the buffer is the array [block, layer, bs*row]
    rng = np.random.Generator(np.random.PCG64(77))
    bs, row, L, nblk = 4, 16, 3, 12
    pools = [rng.integers(0, 256, size=nblk * bs * row, dtype=np.uint8) for _ in range(L)]
    tabs = [np.array([7, 2, 9], np.int32), np.array([0, 11], np.int32)]
    count = [3 * bs, 2 * bs]
    nfb = oracle.fullblock_count(bs, None, count)
    fb = oracle.fullblock_bytes(bs, L, (row,))
    assert nfb == 5 and fb == L * bs * row
    buf = np.full(nfb * fb, 0x77, dtype=np.uint8)
    for l in range(L):
        oracle.pool_to_fullblocks(bs, L, (row,), None, count, tabs, l, [pools[l]], buf)
    flat = np.concatenate(tabs)
    want = np.stack([np.stack([pools[l].reshape(nblk, bs * row)[flat[f]] for l in range(L)]) for f in range(nfb)])
    assert buf.tobytes() == want.tobytes()
    # and layer l of that buffer, taken block by block, is exactly the dense transfer buffer of layer l
    for l in range(L):
        dense = buf.reshape(nfb, L, bs * row)[:, l, :].reshape(-1)
        assert dense.tobytes() == oracle.pack(bs, (row,), count, tabs, [pools[l]]).tobytes()
        a = np.zeros(nblk * bs * row, np.uint8)
        b = np.zeros(nblk * bs * row, np.uint8)
        oracle.fullblocks_to_pool(bs, L, (row,), None, count, tabs, l, buf, [a])
        oracle.unpack(bs, (row,), count, tabs, dense, [b])
        assert a.tobytes() == b.tobytes()
    # (2) ragged ranges, several planes: per-byte brute force, sentinel outside the ranges
    for kw in TINY:
        w = W.tiny(**dict(kw, n_layers=3))
        bs, rows, L = w.layout.block_tokens, w.layout.row_bytes, 3
        for first, count in ((np.zeros_like(w.hit), w.hit), (w.hit, w.app), (np.zeros_like(w.hit), w.hit + w.app)):
            nfb = oracle.fullblock_count(bs, first, count)
            fb = oracle.fullblock_bytes(bs, L, rows)
            lb = fb // L
            assert lb == bs * sum(rows)
            pools = [W.fill_pool(w, l, "src") for l in range(L)]
            buf = np.full(nfb * fb + 8, 0x5A, dtype=np.uint8)
            for l in range(L):
                oracle.pool_to_fullblocks(bs, L, rows, first, count, w.src.tables, l, pools[l], buf)
            ref = np.full(nfb * fb + 8, 0x5A, dtype=np.uint8)
            f = 0
            for r in range(len(count)):
                if int(count[r]) == 0:
                    continue
                b0, b1 = int(first[r]) // bs, (int(first[r]) + int(count[r]) - 1) // bs
                for b in range(b0, b1 + 1):
                    for wi in range(bs):
                        t = b * bs + wi
                        if not (int(first[r]) <= t < int(first[r]) + int(count[r])):
                            continue
                        for l in range(L):
                            po = 0
                            for p, row in enumerate(rows):
                                src_off = (int(w.src.tables[r][b]) * bs + wi) * row
                                dst_off = f * fb + l * lb + po + wi * row
                                ref[dst_off:dst_off + row] = pools[l][p][src_off:src_off + row]
                                po += bs * row
                    f += 1
            assert f == nfb
            assert buf.tobytes() == ref.tobytes(), kw
            # (3) load it back into other tables: equals the Layer-Block scatter of the same rows
            for l in range(L):
                got = W.sentinel_pool(w, "dst")
                oracle.fullblocks_to_pool(bs, L, rows, first, count, w.dst.tables, l, buf, got)
                x = oracle.pack_range(bs, rows, first, count, w.src.tables, pools[l])
                exp = W.sentinel_pool(w, "dst")
                oracle.unpack_range(bs, rows, first, count, w.dst.tables, x, exp)
                for u, v in zip(got, exp):
                    assert u.tobytes() == v.tobytes(), kw


def pin_stream_layers():
    """Layer-wise load from dense host buffers (Section 4.1): layer l comes from host buffer
    l mod H and is what slot l mod S holds when layer l is computed, whatever S and H are.
    Every payload byte carries its layer's tag; H, S and L are pairwise different where it matters."""
    L = 5
    w = W.tiny(seed=41, n_requests=4, block_tokens=8, row_bytes=(32,), pool_blocks=48, max_tokens=50, n_layers=L)
    n = oracle.payload_bytes(w.hit, w.layout.row_bytes)
    layers = [np.full(n, 0x10 + l, dtype=np.uint8) for l in range(L)]   # layer tag in every byte
    mask = brute_hit_mask(8, 32, w.hit, w.dst.tables, w.dst.pool_blocks)
    for S, H in ((1, 2), (2, 2), (5, 2), (2, 3), (3, 1)):
        # host slot h is refilled with layer l's payload just before layer l is loaded
        host = [np.zeros(n, np.uint8) for _ in range(H)]
        slots = [W.sentinel_pool(w, "dst", 0xEE) for _ in range(S)]
        seen = 0
        gen = oracle.stream_layers(8, w.layout.row_bytes, w.hit, w.dst.tables, host, L, slots)
        host[0][:] = layers[0]
        for l in range(L):
            ll, s, planes = next(gen)
            assert (ll, s) == (l, l % S)
            assert planes[0] is slots[l % S][0]
            assert np.all(planes[0][mask] == 0x10 + l)       # the layer being computed is the one resident
            assert np.all(planes[0][~mask] == 0xEE)
            for k in range(S):                                # the other slots hold the layers loaded before
                if k != l % S:
                    older = [m for m in range(l) if m % S == k]
                    want = 0x10 + older[-1] if older else 0xEE
                    assert np.all(slots[k][0][mask] == want), (S, H, l, k)
            if l + 1 < L:
                host[(l + 1) % H][:] = layers[l + 1]
            seen += 1
        assert seen == L
        assert next(gen, None) is None


def pin_stream_fullblocks():
    """Layer-wise load with the storage layout as its source (Appendix A.5: a Full Block is the
    concatenation of a block's Layer Blocks; Section 4.1: layer l's cache is resident when layer l
    is computed).  Expected slot contents are written out with NumPy reshapes of that sentence on
    whole blocks whose bytes carry (block, layer) tags; ragged ranges are checked against the
    dense path (store into Full Blocks, then stream the dense layers)."""
    # (1) whole blocks, two planes, tags: byte (f, l, *) of the buffer is 1 + f * L + l
    bs, rows, L, nblk = 4, (16, 32), 4, 10
    lb = bs * sum(rows)
    tabs = [np.array([7, 2, 9], np.int32), np.array([0, 5], np.int32)]
    count = [3 * bs, 2 * bs]
    flat = np.concatenate(tabs)
    nfb = flat.size
    f_idx, l_idx = np.meshgrid(np.arange(nfb), np.arange(L), indexing="ij")
    tags = (1 + f_idx * L + l_idx).astype(np.uint8)
    blocks = np.repeat(tags.reshape(nfb, L, 1), lb, axis=2)
    # make the bytes inside a Layer Block distinct as well (plane span, row), keeping the tag in the high bits
    inner = (np.arange(lb) % 5).astype(np.uint8)
    blocks = (blocks * np.uint8(5) + inner[None, None, :]).astype(np.uint8)
    buf = np.ascontiguousarray(blocks.reshape(-1))
    for S in (1, 2, 3, L):
        for run in (0, 3):
            slots = [[np.full(nblk * bs * r, 0xEE, np.uint8) for r in rows] for _ in range(S)]
            seen = []
            for l, s, planes in oracle.stream_layers_fullblocks(bs, L, rows, None, count, tabs, buf, slots, run_layers=run):
                assert s == l % S and all(a is b for a, b in zip(planes, slots[s]))
                seen.append(l)
                for k in range(S):
                    older = [m for m in range(l + 1) if m % S == k]
                    off = 0
                    for p, row in enumerate(rows):
                        want = np.full((nblk, bs * row), 0xEE, np.uint8)
                        if older:
                            # plane p's span of layer older[-1]'s Layer Block of every block, block by block
                            want[flat] = blocks[:, older[-1], off:off + bs * row]
                        assert slots[k][p].tobytes() == want.tobytes(), (S, run, l, k, p)
                        off += bs * row
            assert seen == list(range(run or L)), (S, run)
    # (2) ragged ranges and every kind of table: the same observables as the dense path
    for kw in TINY:
        L = 3
        w = W.tiny(**dict(kw, n_layers=L))
        bs, rows = w.layout.block_tokens, w.layout.row_bytes
        for first, count in ((np.zeros_like(w.hit), w.hit), (w.hit, w.app)):
            nfb = oracle.fullblock_count(bs, first, count)
            fb = oracle.fullblock_bytes(bs, L, rows)
            pools = [W.fill_pool(w, l, "src") for l in range(L)]
            buf = np.full(nfb * fb, 0x33, np.uint8)
            dense = []
            for l in range(L):
                oracle.pool_to_fullblocks(bs, L, rows, first, count, w.src.tables, l, pools[l], buf)
                dense.append(oracle.pack_range(bs, rows, first, count, w.src.tables, pools[l]))
            for S in (1, 2, L):
                a = [W.sentinel_pool(w, "dst") for _ in range(S)]
                b = [W.sentinel_pool(w, "dst") for _ in range(S)]
                n = 0
                for l, s, planes in oracle.stream_layers_fullblocks(bs, L, rows, first, count, w.dst.tables, buf, a):
                    oracle.unpack_range(bs, rows, first, count, w.dst.tables, dense[l], b[l % S])
                    assert s == l % S
                    for k in range(S):
                        for u, v in zip(a[k], b[k]):
                            assert u.tobytes() == v.tobytes(), (kw, S, l, k)
                    n += 1
                assert n == L


PINS = [pin_stream_fullblocks, pin_stream_layers, pin_full_blocks, pin_ranges, pin_brute_force, pin_exhaustive_permutations, pin_round_trip, pin_byte_conservation,
        pin_memcpy_and_take, pin_permutation_algebra, pin_closed_form_fill, pin_threads_agree]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()


# --------------------------------------------------------------------------
# preconditions
# --------------------------------------------------------------------------

def test_check_preconditions():
    bs, pool = 4, 10
    ok = [np.array([1, 2, 3], np.int32), np.array([5], np.int32)]
    assert oracle.check(bs, pool, [9, 2], [1, 2], ok, scatter=True) == oracle.OK
    # table too short for hit + appended tokens (9 + 4 tokens need 4 blocks)
    assert oracle.check(bs, pool, [9, 2], [4, 2], ok, scatter=False) == oracle.E_TABLE
    bad = [np.array([1, 2, 10], np.int32), np.array([5], np.int32)]
    assert oracle.check(bs, pool, [9, 2], [1, 2], bad, scatter=False) == oracle.E_BLOCK
    neg = [np.array([1, -1, 3], np.int32), np.array([5], np.int32)]
    assert oracle.check(bs, pool, [9, 2], [1, 2], neg, scatter=False) == oracle.E_BLOCK
    dup = [np.array([1, 2, 3], np.int32), np.array([2], np.int32)]
    assert oracle.check(bs, pool, [9, 2], [1, 2], dup, scatter=False) == oracle.OK   # gather may alias
    assert oracle.check(bs, pool, [9, 2], [1, 2], dup, scatter=True) == oracle.E_DUP
    # a block that only holds appended rows receives nothing, so it cannot alias
    tail = [np.array([1, 2, 3], np.int32), np.array([5, 3], np.int32)]
    assert oracle.check(bs, pool, [8, 2], [4, 6], tail, scatter=True) == oracle.OK


def test_empty_batch_and_zero_hits():
    x = oracle.pack(4, (16,), [], [], [np.zeros(64, np.uint8)])
    assert x.size == 0
    pool = np.arange(4 * 4 * 16, dtype=np.uint8)
    x = oracle.pack(4, (16,), [0, 3, 0], [np.array([0], np.int32), np.array([2], np.int32),
                                          np.zeros(0, np.int32)], [pool])
    assert x.tobytes() == pool[2 * 4 * 16: 2 * 4 * 16 + 3 * 16].tobytes()


# --------------------------------------------------------------------------
# layer-wise streaming: same observables for any number of resident slots
# --------------------------------------------------------------------------

def test_stream_layers_run_layers_beyond_buffer():
    """run_layers only shortens the run: the layers it does load are those of the full run."""
    w = W.tiny(seed=43, n_requests=2, block_tokens=4, row_bytes=(16,), pool_blocks=16, max_tokens=20, n_layers=4)
    bs, rows, L = 4, (16,), 4
    nfb = oracle.fullblock_count(bs, None, w.hit)
    buf = W.random_payload(w, 3, nfb * oracle.fullblock_bytes(bs, L, rows))
    full = [W.sentinel_pool(w, "dst")]          # S = 1
    part = [W.sentinel_pool(w, "dst")]
    got_full = [planes[0].copy() for _, _, planes in
                oracle.stream_layers_fullblocks(bs, L, rows, None, w.hit, w.dst.tables, buf, full)]
    got_part = [planes[0].copy() for _, _, planes in
                oracle.stream_layers_fullblocks(bs, L, rows, None, w.hit, w.dst.tables, buf, part, run_layers=2)]
    assert len(got_full) == 4 and len(got_part) == 2
    for a, b in zip(got_full, got_part):
        assert a.tobytes() == b.tobytes()


# --------------------------------------------------------------------------
# planted mistakes: each must trip at least one pin
# --------------------------------------------------------------------------

MUTANTS = [
    ("swap div and mod", r"tables\[r\]\[t / bs\] \* bs \+ t % bs", "tables[r][t % bs] * bs + t / bs"),
    ("drop row in block", r"\* bs \+ t % bs;", "* bs;"),
    ("block stride off by one", r"tables\[r\]\[t / bs\] \* bs", "tables[r][t / bs] * (bs + 1)"),
    ("request offset uses row count only", r"off \+= \(uint64_t\)hit\[r\] \* row;", "off += (uint64_t)hit[r];"),
    ("plane base forgets T", r"base \+= T \* row;", "base += row;"),
    ("hit loop one short", r"t < hit\[r\]; \+\+t", "t + 1 < hit[r]; ++t"),
    ("row loop one short", r"j < row; \+\+j", "j + 1 < row; ++j"),
    ("xfer index transposed", r"xfer\[off \+ t \* row \+ j\]", "xfer[off + j * hit[r] + t]"),
    ("payload counts one plane", r"bytes \+= T \* \(uint64_t\)row_bytes\[p\];", "bytes = T * (uint64_t)row_bytes[p];"),
    ("range: first token dropped", r"uint64_t t = \(first \? first\[r\] : 0\) \+ k;", "uint64_t t = k;"),
    ("range: buffer indexed by request token", r"xfer\[off \+ k \* row \+ j\]", "xfer[off + t * row + j]"),
    ("range: request offset counts skipped tokens", r"off \+= \(uint64_t\)count\[r\] \* row;",
     "off += ((uint64_t)count[r] + (first ? first[r] : 0)) * row;"),
    ("range: plane base from the wrong total", r"uint64_t T = sum_u32\(n_req, count\);",
     "uint64_t T = sum_u32(n_req, first ? first : count);"),
    ("range: loop one short", r"k < count\[r\]; \+\+k", "k + 1 < count[r]; ++k"),
    ("full block: layer stride is the full block", r"\(uint64_t\)layer \* lb \+ plane_off", "(uint64_t)layer * fb + plane_off"),
    ("full block: plane offset forgets block size", r"plane_off \+= \(uint64_t\)bs \* row;", "plane_off += row;"),
    ("full block: block index not rebased", r"f_base \+ \(t / bs - t0 / bs\)", "f_base + t / bs"),
    ("full block: request base counts tokens", r"f_base \+= \(t0 \+ count\[r\] - 1\) / bs - t0 / bs \+ 1;", "f_base += (count[r] + bs - 1) / bs;"),
    ("full block: row in block dropped", r"plane_off \+ w \* row;", "plane_off + k * row;"),
    ("full block: size counts one plane", r"lb \+= \(uint64_t\)bs \* row_bytes\[p\];\n    return", "lb = (uint64_t)bs * row_bytes[p];\n    return"),
]


def _battery_against(so_path):
    """Run every pin against another build of the oracle; exit code 1 if one trips."""
    with KO.use_library(so_path):
        for pin in PINS:
            try:
                pin()
            except (AssertionError, ValueError, RuntimeError, IndexError):
                return 1
    return 0


@pytest.mark.parametrize("name,pat,rep", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, pat, rep):
    src = open(KO._SRC).read()
    mutated, n = re.subn(pat, rep, src)
    assert n >= 1, "mutation pattern no longer matches the oracle source"
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "m.c")
        so = os.path.join(d, "m.so")
        open(c, "w").write(mutated)
        subprocess.check_call(["gcc", "-std=c99", "-O1", "-w", "-fPIC", "-shared", "-o", so, c])
        # a planted indexing mistake may write out of bounds, so the battery
        # runs in a child process; a crash there also counts as noticed
        code = ("import sys; sys.path.insert(0, %r); sys.path.insert(0, %r); "
                "import test_oracle_pins as t; sys.exit(t._battery_against(%r))"
                % (root, os.path.join(root, "tests"), so))
        rc = subprocess.run([sys.executable, "-c", code], capture_output=True).returncode
        assert rc != 0, f"no pin noticed: {name}"


# The Python layer of the oracle (the per-layer compositions and the request sharding) gets the
# same treatment: mistakes planted in a copy of kvl_oracle.py, the battery run against the copy.
PY_MUTANTS = [
    ("full blocks: slot not wrapped", "stream_layers_fullblocks", "s = l % S", "s = l"),
    ("full blocks: slot one ahead", "stream_layers_fullblocks", "s = l % S", "s = (l + 1) % S"),
    ("full blocks: always layer 0", "stream_layers_fullblocks", "tables, l, blocks", "tables, 0, blocks"),
    ("full blocks: layer one ahead", "stream_layers_fullblocks", "tables, l, blocks", "tables, (l + 1) % n_layers, blocks"),
    ("full blocks: run_layers ignored", "stream_layers_fullblocks", "range(run_layers or n_layers)", "range(n_layers)"),
    ("full blocks: yields slot 0", "stream_layers_fullblocks", "yield l, s, dev_slots[s]", "yield l, s, dev_slots[0]"),
    ("full blocks: loads into slot 0", "stream_layers_fullblocks", "l, blocks, dev_slots[s])", "l, blocks, dev_slots[0])"),
    ("dense: H and S swapped", "stream_layers", "H, S = len(host_layers), len(dev_slots)", "S, H = len(host_layers), len(dev_slots)"),
    ("dense: host slot by S", "stream_layers", "host_layers[l % H]", "host_layers[l % S]"),
    ("dense: host slot fixed", "stream_layers", "host_layers[l % H]", "host_layers[0]"),
    ("dense: slot by H", "stream_layers", "s = l % S", "s = l % H"),
    ("dense: yields slot 0", "stream_layers", "yield l, s, dev_slots[s]", "yield l, s, dev_slots[0]"),
    ("sharding: ranges lose a request", "_ranges", "int(cuts[i + 1]))", "int(cuts[i + 1]) - 1)"),
    ("payload of the first plane only", "payload_bytes", "rb.size, rbp))", "1, rbp))"),
    ("full blocks: count ignores the first token", "fullblock_count", "c.size, fp, cp))", "c.size, None, cp))"),
]


def _mutate_function(src, func, old, new):
    """Replace `old` by `new` inside the top-level function `func` of the source text only."""
    start = src.index("\ndef %s(" % func)
    end = src.find("\ndef ", start + 1)
    end = len(src) if end < 0 else end
    body = src[start:end]
    assert body.count(old) >= 1, "mutation pattern no longer matches the oracle source"
    return src[:start] + body.replace(old, new) + src[end:]


def _battery_against_python(py_path):
    """Run every pin with the oracle's Python layer replaced by another version of its source."""
    code = compile(open(py_path).read(), KO.__file__, "exec")
    exec(code, KO.__dict__)                       # same module object, so paths and the C library stay the real ones
    for name in list(vars(oracle)):
        if name in KO.__dict__ and callable(KO.__dict__[name]):
            setattr(oracle, name, KO.__dict__[name])
    for pin in PINS:
        try:
            pin()
        except (AssertionError, ValueError, RuntimeError, IndexError, TypeError, StopIteration):
            return 1
    return 0


def _run_python_battery(source_text):
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    with tempfile.TemporaryDirectory() as d:
        path = os.path.join(d, "mutant.py")
        open(path, "w").write(source_text)
        code = ("import sys; sys.path.insert(0, %r); sys.path.insert(0, %r); "
                "import test_oracle_pins as t; sys.exit(t._battery_against_python(%r))"
                % (root, os.path.join(root, "tests"), path))
        return subprocess.run([sys.executable, "-c", code], capture_output=True).returncode


def test_python_battery_passes_unmutated():
    """The harness itself: the untouched source, swapped in the same way, passes every pin."""
    assert _run_python_battery(open(KO.__file__).read()) == 0


@pytest.mark.parametrize("name,func,old,new", PY_MUTANTS, ids=[m[0] for m in PY_MUTANTS])
def test_planted_python_mistake_is_caught(name, func, old, new):
    assert _run_python_battery(_mutate_function(open(KO.__file__).read(), func, old, new)) != 0, \
        f"no pin noticed: {name}"
