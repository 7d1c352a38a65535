"""Submission-cost study for the host-buffer load path (needs an MI355X):

    python -m paper_2602_21548_amd.h2d_study [--requests N]

Section 5.2 of the paper observes that a copy engine fed many small copies is bound
by the per-copy submission cost (5-7 us per cudaMemcpyAsync on its hardware, against
about 1 us for an RDMA work request).  This prints what the same question looks
like on this machine for one layer of the streamed MLA workload: one copy per Layer
Block, chunked copies through a staging ring at several chunk sizes, and the scatter
kernel reading the pinned buffer itself.
"""
from __future__ import annotations

import argparse
import time

import torch

import kvl_workloads as W

from . import binding as K


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=0, help="requests of the workload (0: all 128)")
    args = ap.parse_args()
    dev = torch.device("cuda:0")
    w = W.config(5, n_requests=args.requests or None)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    lay = K.make_layout(L, bs, rows, w.dst.pool_blocks)
    plan = K.kvl_plan(lay, w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
    n = plan.payload_bytes
    host = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    host.numpy()[:] = 7
    pool = [torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device=dev) for r in rows]
    cs, ks = torch.cuda.Stream(), torch.cuda.Stream()
    big = torch.empty(min(n, 1 << 30), dtype=torch.uint8, device=dev)
    peak = K.kvl_measure_h2d_peak(host[:big.numel()], big, reps=5, stream=cs)
    del big
    print(f"workload: one layer of {w.name}, {w.n_requests} requests, {n / 1e9:.3f} GB payload, "
          f"{plan.n_units} Layer-Block descriptors of up to {bs * rows[0]} bytes")
    print(f"host link peak (1 GiB pinned hipMemcpyAsync): {peak:.2f} GB/s\n")
    print(f"{'method':44s} {'copies':>8s} {'GB/s':>8s} {'of peak':>8s} {'enqueue us/copy':>16s}")

    def timed(fn, streams):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        copies = fn()
        t1 = time.perf_counter()
        for s in streams:
            s.synchronize()
        t2 = time.perf_counter()
        return copies, n / (t2 - t0) / 1e9, (t1 - t0) * 1e6 / max(1, copies)

    best = None
    for _ in range(2):
        best = timed(lambda: K.kvl_h2d_blockwise_layer(plan, host, pool, stream=cs), [cs])
    c, g, us = best
    print(f"{'one hipMemcpyAsync per Layer Block':44s} {c:8d} {g:8.2f} {g / peak:8.1%} {us:16.2f}")
    for mb in (1, 2, 4, 8, 16, 32, 64, 128, 256):
        chunk = mb << 20
        if chunk < bs * max(rows):
            continue
        staging = torch.empty(4 * chunk, dtype=torch.uint8, device=dev)
        copies = len(plan.chunks(chunk))
        res = None
        for _ in range(2):
            res = timed(lambda: (K.kvl_h2d_unpack_layer(plan, host, staging, chunk, pool, cs, ks), copies)[1], [ks, cs])
        c, g, us = res
        print(f"{'staging ring, chunk ' + str(mb) + ' MiB x 4 slots':44s} {c:8d} {g:8.2f} {g / peak:8.1%} {us:16.2f}")
        del staging
    res = None
    for _ in range(2):
        res = timed(lambda: (K.kvl_unpack_layer(plan, host, pool, stream=ks), 1)[1], [ks])
    c, g, us = res
    print(f"{'scatter kernel reads pinned memory (0 copies)':44s} {0:8d} {g:8.2f} {g / peak:8.1%} {us:16.2f}")
    plan.destroy()


if __name__ == "__main__":
    main()
