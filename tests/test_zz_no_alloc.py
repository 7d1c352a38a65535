"""kvl_unpack_layer_noalloc, the scatter for callers that cannot allocate: its result in the pool
must be, byte for byte, that of kvl_plan + kvl_unpack_layer (and of the oracle), on calls in a
row that share the library's fixed descriptor array, the later ones with smaller inputs.

Collected last on purpose (the file name): the entry point keeps state per process, and a
failure here must not hide the tests of the paper's path.
"""
import numpy as np
import pytest
import torch

import kvl_workloads as W
import oracle
import paper_2602_21548_amd as K
from gpu_util import dev_plan, planes_to_dev, same_bytes, to_dev, to_host


def _layout(w):
    return K.make_layout(w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes, w.dst.pool_blocks)


def _both_ways(w, flags=0, stream=None, seed=0):
    """Scatter one random payload with the plan-based entry point and with the no-alloc one."""
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    zero = np.zeros_like(w.hit)
    if flags & K.KVL_TOKENS_APPEND:
        first, count = w.hit, w.app
    elif flags & K.KVL_TOKENS_ALL:
        first, count = zero, w.hit + w.app
    else:
        first, count = zero, w.hit
    n = oracle.payload_bytes(count, rows)
    x = W.random_payload(w, seed, n)
    want = W.sentinel_pool(w, "dst")
    oracle.unpack_range(bs, rows, first, count, w.dst.tables, x, want, threads=8)
    d_x = to_dev(x) if n else torch.zeros(16, dtype=torch.uint8, device="cuda")
    # the existing entry point
    plan = dev_plan(w, "dst", K.KVL_SCATTER | flags)
    assert plan.payload_bytes == n
    ref = planes_to_dev(W.sentinel_pool(w, "dst"))
    K.kvl_unpack_layer(plan, d_x, ref, stream)
    # the one that allocates nothing
    got = planes_to_dev(W.sentinel_pool(w, "dst"))
    torch.cuda.synchronize()
    K.kvl_unpack_layer_noalloc(_layout(w), w.hit, w.app, w.dst.tables, flags, d_x, got, stream)
    torch.cuda.synchronize()
    for p, (a, b, c) in enumerate(zip(got, ref, want)):
        assert same_bytes(to_host(a), to_host(b)), f"plane {p}: differs from kvl_unpack_layer"
        assert same_bytes(to_host(a), c), f"plane {p}: differs from the oracle"
    plan.destroy()
    return n


@pytest.mark.gpu
def test_two_calls_in_a_row_second_smaller():
    big = W.config(3, n_requests=12, token_scale=1 / 16)          # about 400 descriptors of 72 KiB
    small = W.tiny(231, 5, 16, (48,), 64, 90)
    n_big = _both_ways(big, seed=1)
    n_small = _both_ways(small, seed=2)                            # leaves most of the array holding the first call's descriptors
    assert n_small < n_big
    _both_ways(big, seed=3)                                        # and a larger one again


@pytest.mark.gpu
def test_shapes_ranges_and_streams():
    side = torch.cuda.Stream()
    cases = [
        (W.config(1), 0),
        (W.config(2, n_requests=7, token_scale=1 / 32), 0),                       # two planes
        (W.config(4, n_requests=12, token_scale=1 / 32), 0),                      # 656-byte rows, fragmented tables
        (W.tiny(232, 9, 1, (1152,), 3000, 300), 0),                               # token-granular: the flat kernel
        (W.tiny(233, 4, 3, (5,), 60, 40), 0),                                     # odd rows: the byte kernel
        (W.tiny(234, 7, 4, (32, 16), 200, 60, kind="runs"), K.KVL_NO_MERGE),
        (W.from_trace(32, 6), K.KVL_TOKENS_APPEND),
        (W.from_trace(32, 6), K.KVL_TOKENS_ALL),
    ]
    for i, (w, flags) in enumerate(cases):
        _both_ways(w, flags, stream=side if i % 2 else None, seed=10 + i)


@pytest.mark.gpu
def test_back_to_back_on_two_streams_without_a_host_sync():
    """The second call must not overwrite the descriptors while the first call's kernel reads them."""
    a = W.config(3, n_requests=12, token_scale=1 / 16)
    b = W.config(4, n_requests=12, token_scale=1 / 32)
    outs = []
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for w, s, seed in ((a, streams[0], 5), (b, streams[1], 6), (a, streams[1], 7), (b, streams[0], 8)):
        rows = w.layout.row_bytes
        n = oracle.payload_bytes(w.hit, rows)
        x = W.random_payload(w, seed, n)
        want = W.sentinel_pool(w, "dst")
        oracle.unpack(w.layout.block_tokens, rows, w.hit, w.dst.tables, x, want, threads=8)
        d_x, got = to_dev(x), planes_to_dev(W.sentinel_pool(w, "dst"))
        torch.cuda.synchronize()
        outs.append((d_x, got, want, w, s))
    for d_x, got, want, w, s in outs:                              # four calls enqueued with no sync between them
        K.kvl_unpack_layer_noalloc(_layout(w), w.hit, w.app, w.dst.tables, 0, d_x, got, s)
    torch.cuda.synchronize()
    for d_x, got, want, w, s in outs:
        for a_, b_ in zip(got, want):
            assert same_bytes(to_host(a_), b_)


@pytest.mark.gpu
def test_errors_and_empty_batches():
    w = W.tiny(235, 4, 16, (48,), 64, 90)
    lay = _layout(w)
    n = oracle.payload_bytes(w.hit, w.layout.row_bytes)
    d_x = torch.zeros(n, dtype=torch.uint8, device="cuda")
    pool = planes_to_dev(W.sentinel_pool(w, "dst"))
    with pytest.raises(K.KvlError) as e:                           # transfer buffer too small
        K.kvl_unpack_layer_noalloc(lay, w.hit, w.app, w.dst.tables, 0, d_x[:n - 16], pool)
    assert e.value.code == K.KVL_ESPACE
    with pytest.raises(K.KvlError) as e:                           # a plan flag that is not the caller's to give
        K.kvl_unpack_layer_noalloc(lay, w.hit, w.app, w.dst.tables, K.KVL_GATHER, d_x, pool)
    assert e.value.code == K.KVL_EINVAL
    dup = [t.copy() for t in w.dst.tables]
    dup[1][0] = dup[0][0]
    with pytest.raises(K.KvlError) as e:                           # validation is kvl_plan's
        K.kvl_unpack_layer_noalloc(lay, w.hit, w.app, dup, 0, d_x, pool)
    assert e.value.code == K.KVL_EALIAS
    # more descriptors than the fixed array holds: a clear error, nothing enqueued
    R, bs = 2, 1
    per = K.KVL_NOALLOC_MAX_UNITS // 2 + 1
    hit = np.full(R, per, dtype=np.uint32)
    tables = [np.arange(r * per, (r + 1) * per, dtype=np.int32)[::-1].copy() for r in range(R)]   # descending: nothing merges
    big = K.make_layout(1, bs, (16,), R * per)
    d_big = torch.zeros(R * per * 16, dtype=torch.uint8, device="cuda")
    d_pool = [torch.zeros(R * per * 16, dtype=torch.uint8, device="cuda")]
    with pytest.raises(K.KvlError) as e:
        K.kvl_unpack_layer_noalloc(big, hit, np.zeros(R, np.uint32), tables, 0, d_big, d_pool)
    assert e.value.code == K.KVL_ESPACE
    # exactly at the limit it runs
    hit2 = np.array([per - 1, per - 1], dtype=np.uint32)
    rng = np.random.Generator(np.random.PCG64(9))
    x = rng.integers(0, 256, size=int(hit2.sum()) * 16, dtype=np.uint8)
    want = [np.zeros(R * per * 16, np.uint8)]
    oracle.unpack(bs, (16,), hit2, tables, x, want, threads=8)
    K.kvl_unpack_layer_noalloc(big, hit2, np.zeros(R, np.uint32), tables, 0, to_dev(x), d_pool)
    torch.cuda.synchronize()
    assert same_bytes(to_host(d_pool[0]), want[0])
    # empty batches are fine and touch nothing
    K.kvl_unpack_layer_noalloc(lay, [], [], [], 0, d_x, pool)
    K.kvl_unpack_layer_noalloc(lay, np.zeros_like(w.hit), w.app, w.dst.tables, 0, d_x, pool)
    torch.cuda.synchronize()
    for a_, b_ in zip(pool, W.sentinel_pool(w, "dst")):
        assert same_bytes(to_host(a_), b_)


def test_oversized_batch_is_rejected_before_any_device_call():
    """Host logic only (runs without a GPU): the size check comes before the first HIP call."""
    import ctypes as C
    from paper_2602_21548_amd import binding as B
    per = K.KVL_NOALLOC_MAX_UNITS // 2 + 1
    tables = [np.arange(r * per, (r + 1) * per, dtype=np.int32)[::-1].copy() for r in range(2)]
    reqs, n, _keep = B._requests(np.full(2, per, np.uint32), np.zeros(2, np.uint32), tables)
    lay = K.make_layout(1, 1, (16,), 2 * per)
    planes = (C.c_void_p * 1)(0x1000)                              # never dereferenced on this path
    rc = B._lib.kvl_unpack_layer_noalloc(C.byref(lay), reqs, n, 0, C.c_void_p(0x1000), 2 * per * 16, planes, None)
    assert rc == K.KVL_ESPACE
    rc = B._lib.kvl_unpack_layer_noalloc(C.byref(lay), reqs, n, K.KVL_HOST_ONLY, C.c_void_p(0x1000), 2 * per * 16,
                                         planes, None)
    assert rc == K.KVL_EINVAL
