#!/usr/bin/env python3
"""Benchmark of the layer-wise KV-cache load path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4]

The default workload is the largest one that runs device-resident on one GPU (cfg4: 12.2 GB of
cache per layer, 61 layers, 289,870 fully fragmented blocks); it is also the one whose kernels
run furthest below the memory's peak.  Every other workload gets a short run with a roofline
object of its own (`other_configs`).

A step is one batch through the whole device-resident path: kvl_plan for the
decode side and the prefill side, then for every layer kvl_pack_layer (paged
pool -> transfer buffer) and kvl_unpack_layer (transfer buffer -> second paged
pool).  `value` is the rate at which cache bytes arrive in the prefill pool,
layers x payload / step time, with every input resident in HBM.  The two
entry points that take a pinned host buffer (kvl_h2d_unpack_layer,
kvl_stream_layers) are timed after the steps and reported beside it, against
the host-link rate measured in the same run; they never enter `value`.

Prints one JSON line.  The CPU oracle is timed on a bounded sample of the same
workload as a baseline (`cpu_baseline`), not as a target.  Everything here that
touches oracle/ belongs to that CPU leg and --skip-cpu leaves all of it out: the
oracle's timing, the check of what the GPU left behind against the oracle's row
placement, and the timing of the scheduling oracle.  No timed GPU step calls it.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "KV-cache load GB/s per layer (pack, unpack, H2D+unpack) and % of HBM/link peak"
HBM_PEAK_GBPS = 8000.0
WORKLOADS = {
    1: "cfg1 tiny MLA: 2 layers, 4 req x 1000 hit tokens, bs 16, 1152 B rows",
    2: "cfg2 GQA: 32 layers, K and V planes of 2048 B rows, bs 64, 64 req, hit U[16K,64K], append U[256,1024], pool 1.1x, random tables",
    3: "cfg3 MLA: 61 layers, 1152 B rows, bs 64, 128 req, hit lognormal(median 32K, cap 128K), 95% hit, random tables",
    4: "cfg4 fp8 MLA: 61 layers, 656 B opaque rows, bs 64, 256 req, hit U[8K,128K], fully fragmented tables",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_source_hash() -> str:
    h = hashlib.sha256()
    for f in ("kvl_copy_kernels.h",):
        h.update(open(os.path.join(ROOT, "paper_2602_21548_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload_index: int, kernel: str):
    """HBM bytes per launch from the committed counter runs, or None when the
    kernel source has changed since they were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None
    if rec.get("kernel_source_hash") != kernel_source_hash():
        return None
    return rec.get(f"cfg{workload_index}", {}).get(kernel)


def cpu_baseline(index: int, sample_requests: int) -> dict:
    """The oracle, as it stands, on a sample of the workload: one layer of the
    first `sample_requests` requests, pack then unpack, on the host cores.
    sample_requests == 0: as many of the first requests as keep the payload near 6 GB
    (about 10-30 s of single-threaded work for two layers)."""
    import kvl_workloads as W
    import oracle
    if not sample_requests:
        full = W.config(index)
        per_token = sum(full.layout.row_bytes)
        csum = np.cumsum(full.hit.astype(np.int64)) * per_token
        sample_requests = max(1, int(np.searchsorted(csum, 6.5e9)))
        sample_requests = min(sample_requests, full.n_requests)
        del full
    w = W.config(index, n_requests=sample_requests or None)
    sample_requests = w.n_requests
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = W.fill_pool_fast(w, 0, "src")
    dst = W.sentinel_pool(w, "dst")
    n = oracle.payload_bytes(w.hit, rows)
    x = np.empty(n, dtype=np.uint8)
    cores = len(os.sched_getaffinity(0))
    out = {}
    layers = 2                      # the same pools twice: about 10 s of single-thread work on cfg2
    for label, threads in (("single", 1), ("sharded", max(1, min(cores, sample_requests)))):
        t0 = time.perf_counter()
        for _ in range(layers):
            oracle.pack(bs, rows, w.hit, w.src.tables, src, xfer=x, threads=threads)
            oracle.unpack(bs, rows, w.hit, w.dst.tables, x, dst, threads=threads)
        dt = time.perf_counter() - t0
        out[label] = (layers * n / dt / 1e9, threads, dt)
    v, c, dt = out["sharded"]
    return {"value": round(v, 3), "unit": "GB/s", "cores": c, "kind": "oracle",
            "sample": f"{layers} layers of the first {sample_requests} requests of cfg{index} "
                      f"({n / 1e9:.2f} GB payload per layer), pack+unpack, {dt:.1f} s sharded + "
                      f"{out['single'][2]:.1f} s single-threaded",
            "single_thread_value": round(out["single"][0], 3),
            "single_thread_seconds": round(out["single"][2], 2),
            "host_cores_available": cores}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, choices=sorted(WORKLOADS))
    ap.add_argument("--skip-host-link", action="store_true", help="leave out the pinned-host legs")
    ap.add_argument("--skip-cpu", action="store_true", help="leave out the CPU-oracle baseline")
    ap.add_argument("--skip-other-configs", action="store_true", help="leave out the short runs of the other workloads")
    ap.add_argument("--stream-layers", type=int, default=0, help="layers of the streamed leg (0: all 61)")
    ap.add_argument("--cpu-sample-requests", type=int, default=0,
                    help="requests in the CPU sample (0: the first requests up to about 6 GB of payload)")
    ap.add_argument("--only-h2d-study", action="store_true",
                    help="run the submission-cost study of the host-buffer path and print its table (Section 5.2)")
    ap.add_argument("--skip-studies", action="store_true", help="leave out the ceilings and kernel-shape legs")
    ap.add_argument("--only-steps", action="store_true",
                    help="time the steps only: no tail-return, other-config, host-link or CPU legs (for profiler runs)")
    ap.add_argument("--only-host-link", action="store_true",
                    help="run the pinned-host legs only and print their object (for profiler runs)")
    ap.add_argument("--calibration-copy-gib", type=float, default=0.0,
                    help="also launch one plain copy kernel of this size (a known-traffic reference for counter runs)")
    args = ap.parse_args()
    if args.only_steps:
        args.skip_host_link = args.skip_cpu = args.skip_other_configs = args.skip_studies = True
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus must be 1 "
              "(the load path shards by request across GPUs without any collective)", file=sys.stderr)
        return 2

    import torch
    import kvl_workloads as W
    import paper_2602_21548_amd as K

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.only_host_link:
        print(json.dumps({"host_link": host_link_legs(args)}), flush=True)
        return 0
    if args.only_h2d_study:
        h2d_study()
        return 0

    w = W.config(args.config)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    P = len(rows)
    lay_src = K.make_layout(L, bs, rows, w.src.pool_blocks)
    lay_dst = K.make_layout(L, bs, rows, w.dst.pool_blocks)

    # resident-layer windows: layer l lives in slot l % 2 on both sides (layer-wise
    # prefill keeps only a few layers' cache in HBM at a time)
    WIN = min(2, L)
    log(f"[bench] {WORKLOADS[args.config]}")
    t0 = time.perf_counter()
    src, src_tags = [], []
    for s in range(WIN):
        host_planes = W.fill_pool_fast(w, s, "src")
        src_tags.append(row_heads(host_planes, rows))          # kept on the host for the oracle check
        src.append([torch.from_numpy(p).to(dev) for p in host_planes])
        del host_planes
    dst = [[torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device=dev) for r in rows]
           for _ in range(WIN)]
    probe = K.kvl_plan(lay_src, w.hit, w.app, w.src.tables, K.KVL_GATHER | K.KVL_HOST_ONLY)
    payload, T, n_units = probe.payload_bytes, probe.hit_tokens, probe.n_units
    probe.destroy()
    xfer = torch.empty(payload, dtype=torch.uint8, device=dev)
    log(f"[bench] inputs resident after {time.perf_counter() - t0:.1f} s: payload/layer {payload / 1e9:.3f} GB, "
        f"{T} hit tokens, {n_units} descriptors")

    stream = torch.cuda.Stream()
    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731

    def step(events=None):
        """One batch.  events: a list of L (before pack, between, after unpack) event triples."""
        g = K.kvl_plan(lay_src, w.hit, w.app, w.src.tables, K.KVL_GATHER)
        s = K.kvl_plan(lay_dst, w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
        for l in range(L):
            if events is not None:
                events[l][0].record(stream)
            K.kvl_pack_layer(g, src[l % WIN], xfer, stream=stream)
            if events is not None:
                events[l][1].record(stream)
            K.kvl_unpack_layer(s, xfer, dst[l % WIN], stream=stream)
            if events is not None:
                events[l][2].record(stream)
        # no synchronisation here: destroying a plan does not wait for the device, so the host
        # goes on to plan the next batch while this one's kernels run (the timed region as a
        # whole is bracketed by device-wide synchronisations)
        g.destroy()
        s.destroy()

    if args.calibration_copy_gib > 0:
        nb = int(args.calibration_copy_gib * (1 << 30)) // 16 * 16
        ca = torch.full((nb,), 1, dtype=torch.uint8, device=dev)
        cb = torch.empty_like(ca)
        K.kvl_copy_linear(ca, cb, stream=stream)
        stream.synchronize()
        log(f"[bench] calibration copy: kvl_linear_kernel moved {nb} bytes (reads {nb}, writes {nb})")
        del ca, cb
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the events are made before the clock starts; the timed region only records them
    all_events = [[(ev(), ev(), ev()) for _ in range(L)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(all_events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_kernel = [t for row in all_events for t in row]
    ms_per_step = wall * 1e3 / args.steps
    pack_ms = np.array([a.elapsed_time(b) for a, b, _ in per_kernel])
    unpack_ms = np.array([b.elapsed_time(c) for _, b, c in per_kernel])
    value = L * payload / (ms_per_step * 1e-3) / 1e9
    for name, ms in (("pack", pack_ms), ("unpack", unpack_ms)):
        worst = np.argsort(ms)[-4:][::-1]
        log(f"[bench] {name}: median {np.median(ms):.3f} ms; slowest launches (step, layer, ms): "
            + ", ".join(f"({i // L}, {i % L}, {ms[i]:.2f})" for i in worst))

    # plan cost on its own (host work + descriptor upload), outside the timed steps
    t0 = time.perf_counter()
    for _ in range(5):
        K.kvl_plan(lay_src, w.hit, w.app, w.src.tables, K.KVL_GATHER).destroy()
    plan_ms = (time.perf_counter() - t0) * 1e3 / 5

    # every row's placement, checked against the oracle through 8-byte row tags
    last_slot = (L - 1) % WIN              # the transfer buffer and this slot hold the last layer
    verified = None if args.skip_cpu else verify_tags(w, src_tags[last_slot], dst[last_slot], xfer, T)

    ceiling, runtime_copy = copy_ceiling(stream, args.calibration_copy_gib or 4.0)

    def roof(name, ms):
        return roofline_object(args.config, name, ms, payload, ceiling)

    tail = None if args.only_steps else tail_return_leg(w, lay_src, lay_dst, src, dst, stream, L, WIN)
    fused = None if args.only_steps else fused_move_leg(w, lay_src, lay_dst, src, dst, stream, L, WIN, payload)

    roof_pack = roof("kvl_pack_tile_kernel", pack_ms)
    roof_unpack = roof("kvl_unpack_tile_kernel", unpack_ms)
    dominant, other = (roof_pack, roof_unpack) if pack_ms.sum() >= unpack_ms.sum() else (roof_unpack, roof_pack)

    out = {
        "metric": METRIC, "value": round(value, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u8",
        "data": "synthetic",
        "config": {"workload": WORKLOADS[args.config], "layers": L, "requests": w.n_requests,
                   "hit_tokens": T, "payload_bytes_per_layer": payload, "descriptors": n_units,
                   "step": f"kvl_plan x2 + {L} x (kvl_pack_layer + kvl_unpack_layer), inputs resident in HBM; "
                           "the host plans batch k+1 while the kernels of batch k run",
                   "resident_layer_window": WIN},
        "roofline": dominant, "roofline_other": other,
        "pack_payload_gbps": round(payload / (pack_ms.mean() * 1e-3) / 1e9, 1),
        "unpack_payload_gbps": round(payload / (unpack_ms.mean() * 1e-3) / 1e9, 1),
        "tokens_layers_per_s": round(T * L / (ms_per_step * 1e-3), 1),
        "plan_ms": round(plan_ms, 3), "verified_rows_vs_oracle": verified,
        "linear_copy_ceiling_gbps": round(ceiling, 1),
        "runtime_memcpy_d2d_gbps": round(runtime_copy, 1),
        "tail_return": tail, "fused_move": fused,
    }
    del src, dst, xfer
    torch.cuda.empty_cache()

    if not args.skip_other_configs:
        out["other_configs"] = {f"cfg{i}": short_hop(i, check=not args.skip_cpu, linear_ceiling=ceiling)
                                for i in sorted(WORKLOADS) if i != args.config}
    if not args.skip_studies:
        out["ceilings"] = ceilings_leg(stream, roof_pack, roof_unpack, args.config)
        out["kernel_shapes"] = kernel_shapes_leg()
    if not args.skip_host_link:
        out["host_link"] = host_link_legs(args)
    if not args.only_steps:
        out["scheduler"] = scheduler_leg(with_oracle=not args.skip_cpu)
    if not args.skip_cpu:
        log("[bench] timing the CPU oracle on a sample ...")
        out["cpu_baseline"] = cpu_baseline(args.config, args.cpu_sample_requests)
    print(json.dumps(out), flush=True)
    return 0


def roofline_object(config_index: int, kernel: str, ms, payload: int, linear_ceiling: float) -> dict:
    """The roofline entry of one kernel on one workload: algorithmic bytes per launch (every
    payload byte read once and written once) over the average launch time measured with HIP
    events on the stream the kernel ran on."""
    ms = np.asarray(ms, dtype=np.float64)
    avg = float(ms.mean())
    achieved = 2.0 * payload / (avg * 1e-3) / 1e9
    return {"kernel": kernel, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": measured_traffic(config_index, kernel),
            "frac_of_measured_linear_copy": round(achieved / linear_ceiling, 4) if linear_ceiling else None,
            "algorithmic_bytes_per_launch": 2 * payload, "avg_launch_ms": round(avg, 4),
            "median_launch_ms": round(float(np.median(ms)), 4),
            "min_launch_ms": round(float(ms.min()), 4), "launches": int(ms.size)}


def row_heads(host_planes, rows):
    """First 8 bytes of every row of each plane (host arrays, before they go to the device)."""
    return [np.ascontiguousarray(p.reshape(-1, r)[:, :8]).reshape(-1) for p, r in zip(host_planes, rows)]


def verify_tags(w, tag_src, dst_planes, xfer, T) -> int:
    """The fast fill writes (layer, plane, physical row) into the first 8 bytes of
    every pool row.  Packing and unpacking those tags with the CPU oracle says where
    every row must have gone; compare with what the GPU path left behind."""
    import torch
    import oracle
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    tag_rows = tuple(8 for _ in rows)
    want_x = oracle.pack(bs, tag_rows, w.hit, w.src.tables, tag_src, threads=8)
    want_dst = [np.full(w.dst.pool_blocks * bs * 8, 0xA5, dtype=np.uint8) for _ in rows]
    oracle.unpack(bs, tag_rows, w.hit, w.dst.tables, want_x, want_dst, threads=8)
    checked = 0
    off = 0
    for p, r in enumerate(rows):
        got = xfer[off:off + T * r].view(T, r)[:, :8].contiguous().cpu().numpy().reshape(-1)
        if got.tobytes() != want_x[p * T * 8:(p + 1) * T * 8].tobytes():
            raise SystemExit(f"bench: transfer buffer plane {p} differs from the oracle")
        gd = dst_planes[p].view(-1, r)[:, :8].contiguous().cpu().numpy().reshape(-1)
        if gd.tobytes() != want_dst[p].tobytes():
            raise SystemExit(f"bench: destination pool plane {p} differs from the oracle")
        off += T * r
        checked += T + w.dst.pool_blocks * bs
    return checked


def tail_return_leg(w, lay_src, lay_dst, src, dst, stream, L, WIN) -> dict:
    """The hop after each layer's compute on the decode-engine read path: only the appended
    (miss) tokens' cache goes back, prefill pool -> transfer buffer -> decode pool.  A few
    hundred tokens per request, so launches, not bandwidth, set the time."""
    import torch
    import paper_2602_21548_amd as K
    g = K.kvl_plan(lay_dst, w.hit, w.app, w.dst.tables, K.KVL_GATHER | K.KVL_TOKENS_APPEND)
    s = K.kvl_plan(lay_src, w.hit, w.app, w.src.tables, K.KVL_SCATTER | K.KVL_TOKENS_APPEND)
    n, T = g.payload_bytes, g.hit_tokens
    x = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    ms = []
    for rep in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for l in range(L):
            K.kvl_pack_layer(g, dst[l % WIN], x, stream=stream)
            K.kvl_unpack_layer(s, x, src[l % WIN], stream=stream)
        e1.record(stream)
        e1.synchronize()
        if rep:
            ms.append(e0.elapsed_time(e1) / L)
    g.destroy()
    s.destroy()
    per_layer = float(np.mean(ms))
    return {"what": "appended-tail return hop (pack + unpack per layer), same workload",
            "tokens": T, "payload_bytes_per_layer": n, "us_per_layer": round(per_layer * 1e3, 2),
            "payload_gbps": round(n / (per_layer * 1e-3) / 1e9, 1) if n else 0.0}


def scheduler_leg(with_oracle: bool = True) -> dict:
    """Host cost of the request scheduling rules (Section 6.1): one prefill fetch and one decode
    fetch over 8 engines and a queue of 1024 requests drawn from the synthetic 64K agent trace
    (trajectories whose averages reproduce the paper's table of trace statistics)."""
    import kvl_workloads as W
    from paper_2602_21548_amd import sched as S
    rng = np.random.Generator(np.random.PCG64(20260221 + 400))
    trace = W.agent_trace(64)
    pick = rng.choice(trace.traj.size, size=1024, replace=False)
    Q = (trace.context + trace.append)[pick].astype(np.uint64)
    tok = rng.integers(0, 400_000, size=8).astype(np.uint64)
    read_q = rng.integers(0, 300_000, size=8).astype(np.uint64)
    seq = rng.integers(0, 32, size=8).astype(np.uint64)
    free = np.full(8, 6_000_000, dtype=np.uint64)
    # beta: 2 M unfinished tokens per engine, so that the prefill fetch fills the engines and ends
    # part-way through the queue (the queue holds about twice what 8 engines may take)
    alpha, beta = 150_000, 2_000_000
    reps = 50
    t0 = time.perf_counter()
    for _ in range(reps):
        a, _t = S.kvl_sched_pe_fetch(tok, read_q, Q, alpha, beta)
        d = S.kvl_sched_de_fetch(tok, seq, free, Q)[0]
    decisions = sum(e >= 0 for e in a) + sum(e >= 0 for e in d)
    lib_us = (time.perf_counter() - t0) / reps / max(1, decisions) * 1e6
    what = ("Algorithm 1 prefill fetch (beta = 2 M tokens per engine) + decode phase-2 fetch, 8 engines, "
            "1024 queued requests of the 64K agent trace")
    out = {"what": what, "prefill_requests_placed": sum(e >= 0 for e in a),
           "decode_requests_placed": sum(e >= 0 for e in d), "library_us_per_decision": round(lib_us, 3)}
    if not with_oracle:
        return out
    from oracle import sched_oracle as O
    t0 = time.perf_counter()
    oa = O.pe_fetch(tok.tolist(), read_q.tolist(), Q.tolist(), alpha, beta)
    od = O.de_fetch(tok.tolist(), seq.tolist(), free.tolist(), Q.tolist())[0]
    ora_us = (time.perf_counter() - t0) / max(1, decisions) * 1e6
    if a != oa or d != od:
        raise SystemExit("bench: scheduler decisions differ from the oracle")
    out.update({"oracle_us_per_decision": round(ora_us, 3), "decisions_match_oracle": True})
    return out


def fused_move_leg(w, lay_src, lay_dst, src, dst, stream, L, WIN, payload) -> dict:
    """Both pools on this device: the paired plan moves pool to pool in one kernel per layer,
    without the transfer buffer (half the memory traffic of pack + unpack)."""
    import torch
    import paper_2602_21548_amd as K
    g = K.kvl_plan(lay_src, w.hit, w.app, w.src.tables, K.KVL_GATHER)
    s = K.kvl_plan(lay_dst, w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
    m = K.kvl_plan_pair(g, s)
    ms = []
    for rep in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for l in range(L):
            K.kvl_move_layer(m, src[l % WIN], dst[l % WIN], stream=stream)
        e1.record(stream)
        e1.synchronize()
        if rep:
            ms.append(e0.elapsed_time(e1) / L)
    for p in (g, s, m):
        p.destroy()
    per_layer = float(np.mean(ms))
    return {"what": "kvl_move_layer, pool to pool on one device (no transfer buffer), same workload",
            "ms_per_layer": round(per_layer, 4), "delivered_gbps": round(payload / (per_layer * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(2 * payload / (per_layer * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}


def copy_ceiling(stream, gib: float = 4.0):
    """Traffic rate (GB/s, read + write) of a plain 4 GiB device-to-device copy with the
    pack kernel's instruction mix: what a gather with perfect locality could reach here.
    Second value: the same copy done by the HIP runtime's own device-to-device memcpy
    (torch's copy_ of a contiguous byte tensor), as an independent reference."""
    import torch
    import paper_2602_21548_amd as K
    n = int(gib * (1 << 30)) // 16 * 16
    a = torch.full((n,), 1, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    best = 0.0
    for i in range(6):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        K.kvl_copy_linear(a, b, stream=stream)
        e1.record(stream)
        e1.synchronize()
        if i:
            best = max(best, 2.0 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    runtime = 0.0
    with torch.cuda.stream(stream):
        for i in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            b.copy_(a)
            e1.record(stream)
            e1.synchronize()
            if i:
                runtime = max(runtime, 2.0 * n / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return best, runtime


def short_hop(index: int, reps: int = 8, check: bool = True, linear_ceiling: float = 0.0) -> dict:
    """pack + unpack of one resident layer of another workload, timed per launch."""
    import torch
    import kvl_workloads as W
    import paper_2602_21548_amd as K
    dev = torch.device("cuda:0")
    w = W.config(index)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    host_planes = W.fill_pool_fast(w, 0, "src")
    src_tags = row_heads(host_planes, rows)
    src = [torch.from_numpy(p).to(dev) for p in host_planes]
    del host_planes
    dst = [torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device=dev) for r in rows]
    t0 = time.perf_counter()
    g = K.kvl_plan(K.make_layout(L, bs, rows, w.src.pool_blocks), w.hit, w.app, w.src.tables, K.KVL_GATHER)
    s = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
    plan_ms = (time.perf_counter() - t0) * 1e3 / 2
    payload, T = g.payload_bytes, g.hit_tokens
    xfer = torch.empty(payload, dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    pk, up = [], []
    for i in range(reps + 2):
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record(stream)
        K.kvl_pack_layer(g, src, xfer, stream=stream)
        e1.record(stream)
        K.kvl_unpack_layer(s, xfer, dst, stream=stream)
        e2.record(stream)
        e2.synchronize()
        if i >= 2:
            pk.append(e0.elapsed_time(e1))
            up.append(e1.elapsed_time(e2))
    verified = verify_tags(w, src_tags, dst, xfer, T) if check else None
    pm, um = float(np.mean(pk)), float(np.mean(up))
    out = {"workload": WORKLOADS[index], "payload_bytes_per_layer": payload, "hit_tokens": T,
           "pack_ms": round(pm, 4), "unpack_ms": round(um, 4),
           "pack_payload_gbps": round(payload / pm / 1e6, 1), "unpack_payload_gbps": round(payload / um / 1e6, 1),
           "pack_frac_of_hbm_peak": round(2 * payload / pm / 1e6 / HBM_PEAK_GBPS, 4),
           "unpack_frac_of_hbm_peak": round(2 * payload / um / 1e6 / HBM_PEAK_GBPS, 4),
           "tokens_layers_per_s": round(T / ((pm + um) * 1e-3), 1), "verified_rows_vs_oracle": verified,
           "plan_ms": round(plan_ms, 3), "descriptors": g.n_units,
           "roofline": {"pack": roofline_object(index, "kvl_pack_tile_kernel", pk, payload, linear_ceiling),
                        "unpack": roofline_object(index, "kvl_unpack_tile_kernel", up, payload, linear_ceiling)}}
    # pool to pool in one kernel (paired plan), after the hop above has been checked
    m = K.kvl_plan_pair(g, s)
    mv = []
    for i in range(reps + 2):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        K.kvl_move_layer(m, src, dst, stream=stream)
        e1.record(stream)
        e1.synchronize()
        if i >= 2:
            mv.append(e0.elapsed_time(e1))
    m.destroy()
    mm = float(np.mean(mv))
    out["move_ms"] = round(mm, 4)
    out["move_delivered_gbps"] = round(payload / mm / 1e6, 1)
    out["move_frac_of_hbm_peak"] = round(2 * payload / mm / 1e6 / HBM_PEAK_GBPS, 4)
    if payload < (64 << 20):
        out["note"] = "launch- and cache-bound: the payload fits the on-die cache and a launch costs more than the copy"
        # in this regime the host's launch cost is what a HIP graph removes: capture a run of
        # hops (as the layers of one batch would be), replay it
        HOPS = 16

        def hops():
            for _ in range(HOPS):
                K.kvl_pack_layer(g, src, xfer, stream=stream)
                K.kvl_unpack_layer(s, xfer, dst, stream=stream)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(stream):
            with torch.cuda.graph(graph, stream=stream):
                hops()
            res = {}
            for name, fn in (("eager", hops), ("graph", graph.replay)):
                for _ in range(5):
                    fn()
                stream.synchronize()
                t0 = time.perf_counter()
                for _ in range(50):
                    fn()
                stream.synchronize()
                res[name] = (time.perf_counter() - t0) / (50 * HOPS) * 1e6
        out["hop_us_eager"], out["hop_us_hip_graph"] = round(res["eager"], 2), round(res["graph"], 2)
        out["hops_per_graph"] = HOPS
        del graph
        # the same eager hops with plans whose launches are not followed by an event each
        # (KVL_CALLER_SYNCS: the caller synchronises before it destroys them)
        g2 = K.kvl_plan(K.make_layout(L, bs, rows, w.src.pool_blocks), w.hit, w.app, w.src.tables,
                        K.KVL_GATHER | K.KVL_CALLER_SYNCS)
        s2 = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                        K.KVL_SCATTER | K.KVL_CALLER_SYNCS)

        def hops2():
            for _ in range(HOPS):
                K.kvl_pack_layer(g2, src, xfer, stream=stream)
                K.kvl_unpack_layer(s2, xfer, dst, stream=stream)
        for _ in range(5):
            hops2()
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(50):
            hops2()
        stream.synchronize()
        out["hop_us_eager_caller_syncs"] = round((time.perf_counter() - t0) / (50 * HOPS) * 1e6, 2)
        g2.destroy()
        s2.destroy()
        out["host_buffer_load"] = small_host_buffer_load(s, dst, payload, stream)
    g.destroy()
    s.destroy()
    del src, dst, xfer
    torch.cuda.empty_cache()
    return out


def small_host_buffer_load(s, dst, payload, stream) -> dict:
    """The host-buffer load of a layer that is small (a few MB): the time goes into enqueueing,
    not into the link.  The staged form eager, the same captured in a HIP graph, and the
    zero-copy form (one kernel that reads the pinned buffer itself)."""
    import torch
    import paper_2602_21548_amd as K
    host = torch.zeros(payload, dtype=torch.uint8, pin_memory=True)
    chunk = 1 << 20
    staging = torch.empty(2 * chunk, dtype=torch.uint8, device="cuda")

    def staged():
        K.kvl_h2d_unpack_layer(s, host, staging, chunk, dst, stream, stream)

    def zero_copy():
        K.kvl_h2d_unpack_layer(s, host, None, 0, dst, stream, stream)

    staged()
    stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            staged()

    def replay():
        with torch.cuda.stream(stream):
            graph.replay()

    res = {"payload_bytes": payload, "staged": "2 slots of 1 MiB"}
    for name, fn in (("staged_eager", staged), ("staged_hip_graph", replay), ("zero_copy_eager", zero_copy)):
        fn()
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(30):
            fn()
        stream.synchronize()
        us = (time.perf_counter() - t0) / 30 * 1e6
        res[name + "_us_per_layer"] = round(us, 1)
        res[name + "_gbps"] = round(payload / us / 1e3, 2)
    del graph
    return res


def host_link_legs(args) -> dict:
    """kvl_h2d_unpack_layer on one layer and kvl_stream_layers over all layers of
    the streamed MLA workload, against the host-link rate measured here."""
    import torch
    import kvl_workloads as W
    import paper_2602_21548_amd as K
    dev = torch.device("cuda:0")
    w = W.config(5)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    if args.stream_layers:
        L = min(L, args.stream_layers)
    lay = K.make_layout(w.layout.n_layers, bs, rows, w.dst.pool_blocks)
    plan = K.kvl_plan(lay, w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
    payload = plan.payload_bytes
    H, S = w.notes["host_slots"], w.notes["dev_slots"]
    log(f"[bench] host-link legs: pinning {H} x {payload / 1e9:.2f} GB ...")
    host = [torch.empty(payload, dtype=torch.uint8, pin_memory=True) for _ in range(H)]
    rng = np.random.Generator(np.random.PCG64(W.BASE_SEED + 205))
    tile = rng.integers(0, 256, size=1 << 24, dtype=np.uint8)
    for h in host:
        a = h.numpy()
        for pos in range(0, payload, tile.size):
            k = min(tile.size, payload - pos)
            a[pos:pos + k] = tile[:k]
    slots = [[torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device=dev) for r in rows]
             for _ in range(S)]
    chunk = 128 << 20
    staging = torch.empty(4 * chunk, dtype=torch.uint8, device=dev)
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    peak_buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
    peak = K.kvl_measure_h2d_peak(host[0][:1 << 30], peak_buf, reps=5, stream=cs)
    del peak_buf

    # one layer through the host-buffer path
    times = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        K.kvl_h2d_unpack_layer(plan, host[0], staging, chunk, slots[0], cs, ks)
        ks.synchronize()
        cs.synchronize()
        times.append(time.perf_counter() - t0)
    h2d_gbps = payload / min(times) / 1e9

    st = K.kvl_stream_layers(plan, host, slots, staging, chunk, w.notes["compute_us"], cs, ks, ms, n_layers=L)
    busy = stream_under_busy_compute(plan, host, slots, staging, chunk, cs, ks, ms, min(L, 8), peak)
    # the other direction: gather one layer straight into the pinned host buffer (the step that
    # sends a layer's cache on to the decode engine's host buffer)
    gplan = K.kvl_plan(lay, w.hit, w.app, w.dst.tables, K.KVL_GATHER)
    d2h = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        K.kvl_pack_layer(gplan, slots[0], host[1], stream=ks)
        ks.synchronize()
        d2h.append(time.perf_counter() - t0)
    d2h_gbps = payload / min(d2h) / 1e9
    d2h = []
    for _ in range(3):                 # the same gather staged: pack kernels into HBM slots, copy engine out
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        K.kvl_d2h_pack_layer(gplan, slots[0], staging, chunk, host[1], ks, cs)
        ks.synchronize()
        cs.synchronize()
        d2h.append(time.perf_counter() - t0)
    gplan.destroy()
    d2h_staged_gbps = payload / min(d2h) / 1e9
    duplex = duplex_leg(w, lay, plan, host, slots, staging, chunk, cs, ks, ms, min(L, 16), peak)
    # the same 61 layers with the zero-copy form (scatter kernel reads the pinned buffers itself)
    zc = K.kvl_stream_layers(plan, host, slots, None, 0, w.notes["compute_us"], cs, ks, ms, n_layers=L)
    plan.destroy()
    del slots, staging
    torch.cuda.empty_cache()
    fullblocks = full_block_leg(host[0], peak)
    return {
        "full_blocks": fullblocks, "stream_under_hbm_bound_compute": busy, "stream_with_outflow": duplex,
        "workload": "cfg5 streamed MLA: 61 layers x 1152 B rows, 128 req, pinned host buffer -> paged HBM, "
                    "200 us synthetic compute per layer",
        "h2d_peak_gbps": round(peak, 2), "chunk_bytes": chunk, "staging_slots": 4,
        "h2d_unpack_layer_gbps": round(h2d_gbps, 2), "h2d_unpack_frac_of_link": round(h2d_gbps / peak, 4),
        "stream_layers": L, "stream_total_ms": round(st["total_ms"], 2),
        "stream_gbps": round(st["link_gbps"], 2), "stream_frac_of_link": round(st["link_gbps"] / peak, 4),
        "stream_exposed_ms": round(st["exposed_ms"], 2),
        "pack_to_host_layer_gbps": round(d2h_gbps, 2),
        "pack_to_host_staged_layer_gbps": round(d2h_staged_gbps, 2),
        "stream_zero_copy_gbps": round(zc["link_gbps"], 2),
        "stream_zero_copy_frac_of_link": round(zc["link_gbps"] / peak, 4),
        "payload_bytes_per_layer": payload,
    }


def duplex_leg(w, lay, plan, host, slots, staging, chunk, cs, ks, ms, layers, peak) -> dict:
    """The whole loop of layer-wise prefill: while layer l+1 is loaded and layer l computed
    (200 us stand-in), layer l-1 -- hit and appended rows -- is gathered out to pinned host
    memory.  Both directions of the host link carry a layer at a time."""
    import torch
    import paper_2602_21548_amd as K
    out = K.kvl_plan(lay, w.hit, w.app, w.dst.tables, K.KVL_GATHER | K.KVL_TOKENS_ALL)
    out_host = [torch.empty(out.payload_bytes, dtype=torch.uint8, pin_memory=True) for _ in range(2)]
    # few lanes: the process has 4 hardware queues by default, and lanes that share one with each
    # other or with the caller's streams wait for each other (2 + 1 lanes measured 66 GB/s both
    # ways, 2 + 2 lanes 39, 4 + 4 lanes 52)
    out_staging = torch.empty(chunk, dtype=torch.uint8, device="cuda")
    load_staging = staging[:2 * chunk]
    res = {"layers": layers, "out_payload_bytes_per_layer": out.payload_bytes,
           "note": "rates over the whole run; the outflow of the last layer runs after the last load"}
    res["staged_lanes"] = "2 x 128 MiB in, 1 x 128 MiB out"
    for name, stg, ostg, ch in (("staged_both_ways", load_staging, out_staging, chunk), ("zero_copy_both_ways", None, None, 0)):
        st = K.kvl_stream_layers(plan, host, slots, stg, ch, w.notes["compute_us"], cs, ks, ms, n_layers=layers,
                                 out_plan=out, out_host_layers=out_host, out_staging=ostg, out_chunk_bytes=ch)
        res[name] = {"total_ms": round(st["total_ms"], 2), "h2d_gbps": round(st["link_gbps"], 2),
                     "d2h_gbps": round(st["out_gbps"], 2),
                     "both_ways_gbps": round(st["link_gbps"] + st["out_gbps"], 2)}
    out.destroy()
    del out_host, out_staging
    torch.cuda.empty_cache()
    return res


def stream_under_busy_compute(plan, host, slots, staging, chunk, cs, ks, ms, layers, peak) -> dict:
    """The streamed load with the caller's own computation in place of the 200 us stand-in: per
    layer, plain device-to-device copies that keep every compute unit and the HBM busy for about
    50 ms.  Shows what the load keeps of the link, and what it costs the computation, when the
    GPU is not idle."""
    import torch
    import paper_2602_21548_amd as K
    a = torch.full((4 << 30,), 1, dtype=torch.uint8, device="cuda")
    b = torch.empty_like(a)
    reps = 40

    def compute(layer, slot, stream_handle):
        for _ in range(reps):
            K.kvl_copy_linear(a, b, stream=stream_handle)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(ms)
    compute(0, 0, ms.cuda_stream)
    e1.record(ms)
    e1.synchronize()
    alone = e0.elapsed_time(e1)
    res = {"layers": layers, "compute": f"{reps} x 4 GiB device copies per layer on the compute stream",
           "compute_ms_per_layer_alone": round(alone, 2),
           "hw_queues": os.environ.get("GPU_MAX_HW_QUEUES", "runtime default")}
    for name, stg, ch in (("zero_copy", None, 0), ("staged_2_slots", staging[:2 * chunk], chunk)):
        st = K.kvl_stream_layers(plan, host, slots, stg, ch, 0, cs, ks, ms, n_layers=layers,
                                 compute=compute, per_layer_times=True)
        # the last layer's computation runs after every load has finished: leave it out
        busy = (st["t_compute_end"] - st["t_compute_begin"])[:-1]
        res[name] = {"link_gbps": round(st["link_gbps"], 2), "frac_of_link": round(st["link_gbps"] / peak, 4),
                     "compute_ms_per_layer_during_load": round(float(busy.mean()), 2) if len(busy) else None}
    del a, b
    torch.cuda.empty_cache()
    return res


def full_block_leg(pinned: "torch.Tensor", h2d_peak: float) -> dict:
    """Storage layout: 61-layer Full Blocks in pinned host memory (4 requests of the MLA
    workload); every layer loaded into a paged pool, and stored back, by one kernel per layer
    that converts the layout while it crosses the host link."""
    import torch
    import kvl_workloads as W
    import paper_2602_21548_amd as K
    dev = torch.device("cuda:0")
    w = W.config(3, n_requests=4)
    L, bs, rows = w.layout.n_layers, w.layout.block_tokens, w.layout.row_bytes
    s = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                   K.KVL_SCATTER | K.KVL_GATHER | K.KVL_NO_MERGE)
    fb, nfb = s.fullblock_geometry()
    need = fb * nfb
    while need > pinned.numel():                       # fit the pinned buffer the caller already has
        w = W.config(3, n_requests=w.n_requests - 1)
        s.destroy()
        s = K.kvl_plan(K.make_layout(L, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables,
                       K.KVL_SCATTER | K.KVL_GATHER | K.KVL_NO_MERGE)
        fb, nfb = s.fullblock_geometry()
        need = fb * nfb
    buf = pinned[:need]
    pool = [torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device=dev) for r in rows]
    st = torch.cuda.Stream()
    per_layer = s.payload_bytes
    out = {"workload": f"{w.n_requests} requests of cfg3, {nfb} Full Blocks of {fb} bytes ({L} layers x {bs} x {rows[0]} B)",
           "bytes_per_layer": per_layer}
    for name, fn in (("h2d", lambda l: K.kvl_fullblocks_to_pool_layer(s, buf, l, pool, stream=st)),
                     ("d2h", lambda l: K.kvl_pool_to_fullblocks_layer(s, pool, l, buf, stream=st))):
        best = 0.0
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for l in range(L):
                fn(l)
            e1.record(st)
            e1.synchronize()
            best = max(best, per_layer * L / (e0.elapsed_time(e1) * 1e-3) / 1e9)
        out[f"{name}_gbps"] = round(best, 2)
    out["h2d_frac_of_link"] = round(out["h2d_gbps"] / h2d_peak, 4)
    # the same load staged (the runtime's strided copies into 2 slots of 64 MiB, converting kernels there)
    chunk = 64 << 20
    staging = torch.empty(2 * chunk, dtype=torch.uint8, device=dev)
    cs = torch.cuda.Stream()
    best = 0.0
    for rep in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(st)
        for l in range(L):
            K.kvl_h2d_fullblocks_layer(s, buf, l, staging, chunk, pool, cs, st)
        e1.record(st)
        e1.synchronize()
        cs.synchronize()
        best = max(best, per_layer * L / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out["h2d_staged_gbps"] = round(best, 2)
    out["h2d_staged_frac_of_link"] = round(best / h2d_peak, 4)
    best = 0.0
    for rep in range(3):               # and the persist direction, staged
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(st)
        for l in range(L):
            K.kvl_d2h_fullblocks_layer(s, pool, l, staging, chunk, buf, st, cs)
        e1.record(st)
        e1.synchronize()
        cs.synchronize()
        best = max(best, per_layer * L / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    out["d2h_staged_gbps"] = round(best, 2)
    # the streamed load with the storage layout as its source: 61 layers under 200 us of compute each
    slots = [pool, [torch.full_like(p, 0xA5) for p in pool]]
    cs, ks, ms = torch.cuda.Stream(), torch.cuda.Stream(), torch.cuda.Stream()
    stt = K.kvl_stream_layers(s, None, slots, None, 0, 200, cs, ks, ms, n_layers=L, full_blocks=buf)
    out["stream_from_full_blocks_gbps"] = round(stt["link_gbps"], 2)
    out["stream_from_full_blocks_ms"] = round(stt["total_ms"], 2)
    # beside a computation that keeps the GPU busy (2 x 4 GiB device copies per layer): what each
    # form of the load costs that computation
    a = torch.full((4 << 30,), 1, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)

    def compute(layer, slot, stream_handle):
        K.kvl_copy_linear(a, b, stream=stream_handle)
        K.kvl_copy_linear(a, b, stream=stream_handle)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(ms)
    compute(0, 0, ms.cuda_stream)
    e1.record(ms)
    e1.synchronize()
    busy = {"compute_ms_per_layer_alone": round(e0.elapsed_time(e1), 3)}
    for name, stg, ch in (("zero_copy", None, 0), ("staged", staging, chunk)):
        r = K.kvl_stream_layers(s, None, slots, stg, ch, 0, cs, ks, ms, n_layers=L, full_blocks=buf,
                                compute=compute, per_layer_times=True)
        during = (r["t_compute_end"] - r["t_compute_begin"])[:-1]
        busy[name] = {"total_ms": round(r["total_ms"], 1), "compute_ms_per_layer": round(float(during.mean()), 3)}
    out["beside_busy_compute"] = busy
    del a, b
    s.destroy()
    return out


def _time_launches(fn, stream, reps: int = 8, warm: int = 2) -> float:
    """Average duration in ms of `reps` launches of fn() on `stream` (HIP events on that stream)."""
    import torch
    ms = []
    for i in range(reps + warm):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        fn()
        e1.record(stream)
        e1.synchronize()
        if i >= warm:
            ms.append(e0.elapsed_time(e1))
    return float(np.mean(ms))


def ceilings_leg(stream, roof_pack: dict, roof_unpack: dict, config_index: int) -> dict:
    """What the memory of this machine does on reference streams that use the load and store
    instructions and cache policies of the default kernels but no descriptors: a linear copy and
    its read and write halves alone (4 GiB), and a copy with the access shape of cfg4 -- one
    side dense, the other hopping every 41,984 bytes to a pseudo-random block, the two sides 16
    bytes apart in their 128-byte lines -- with the block's address computed, or read from a
    4-byte table entry through the scalar cache as a descriptor is; and that last form once more with
    every hop kept within 16 neighbouring blocks, which shows what the distance of the hops costs."""
    import torch
    import paper_2602_21548_amd as K
    dev = torch.device("cuda:0")
    out = {"unit": "GB/s of memory traffic (bytes read + bytes written)", "peak": HBM_PEAK_GBPS}
    n = 4 << 30
    a = torch.full((n + 128,), 1, dtype=torch.uint8, device=dev)
    b = torch.empty(n, dtype=torch.uint8, device=dev)
    lin = {}
    for name, mode, factor in (("copy", K.KVL_CEILING_COPY, 2.0), ("read_only", K.KVL_CEILING_READ, 1.0),
                               ("write_only", K.KVL_CEILING_WRITE, 1.0)):
        ms = _time_launches(lambda: K.kvl_ceiling_kernel(mode, a, b, n, stream=stream), stream)
        lin[name] = round(factor * n / ms / 1e6, 1)
    ms = _time_launches(lambda: K.kvl_ceiling_kernel(K.KVL_CEILING_COPY, a, b, n, skew_bytes=16, stream=stream), stream)
    lin["copy_source_16_bytes_off_its_lines"] = round(2.0 * n / ms / 1e6, 1)
    r, w = lin["read_only"], lin["write_only"]
    lin["harmonic_mean_of_read_and_write"] = round(2.0 / (1.0 / r + 1.0 / w), 1)
    out["linear_4GiB"] = lin
    del a, b
    torch.cuda.empty_cache()
    # the shape of cfg4: 2^18 blocks of 64 x 656 bytes, the hopping side holds 2^19
    block, k_dense, k_hop, skew = 64 * 656, 18, 19, 16
    payload = (1 << k_dense) * block
    hop = torch.full(((1 << k_hop) * block,), 1, dtype=torch.uint8, device=dev)
    dense = torch.full((payload + 128,), 2, dtype=torch.uint8, device=dev)
    # the table holds the blocks the computed form would visit (u * odd constant mod 2^19)
    table = ((torch.arange(1 << k_dense, dtype=torch.int64, device=dev) * 0x9e3779b1) & ((1 << k_hop) - 1)).to(torch.int32)
    shape = {"block_bytes": block, "blocks": 1 << k_dense, "payload_bytes": payload, "skew_bytes": skew}
    for side, name, src, dst in ((0, "gather", hop, dense), (1, "scatter", dense, hop)):
        for tname, tab in (("computed_address", None), ("table_entry_per_block", table)):
            ms = _time_launches(lambda: K.kvl_ceiling_kernel(K.KVL_CEILING_COPY, src, dst, payload, block_bytes=block,
                                                             hopping_side=side, skew_bytes=skew, hop_blocks_log2=k_hop,
                                                             block_table=tab, stream=stream), stream)
            shape[f"{name}_{tname}"] = round(2.0 * payload / ms / 1e6, 1)
    # the same copy with the hops kept local: the blocks of every 16 consecutive ones (0.7 MB) are
    # permuted among themselves, so only how far a hop goes differs from the table above
    u = torch.arange(1 << k_dense, dtype=torch.int64, device=dev)
    near = ((u // 16) * 16 + (u % 16) * 5 % 16).to(torch.int32)
    for side, name, src, dst in ((0, "gather", hop, dense), (1, "scatter", dense, hop)):
        ms = _time_launches(lambda: K.kvl_ceiling_kernel(K.KVL_CEILING_COPY, src, dst, payload, block_bytes=block,
                                                         hopping_side=side, skew_bytes=skew, hop_blocks_log2=k_hop,
                                                         block_table=near, stream=stream), stream)
        shape[f"{name}_table_entry_hops_within_16_blocks"] = round(2.0 * payload / ms / 1e6, 1)
    del u, near
    out["shape_of_cfg4"] = shape
    if config_index == 4:
        best_g = max(shape["gather_computed_address"], shape["gather_table_entry_per_block"])
        best_s = max(shape["scatter_computed_address"], shape["scatter_table_entry_per_block"])
        out["library_over_shape_ceiling"] = {"pack": round(roof_pack["achieved"] / best_g, 4),
                                             "unpack": round(roof_unpack["achieved"] / best_s, 4)}
    del hop, dense, table
    torch.cuda.empty_cache()
    return out


def kernel_shapes_leg(index: int = 3) -> dict:
    """The kernel forms the library holds, on one layer of cfg3: the default (tiled, one vector
    per lane, one-shot workgroups) against one wavefront per descriptor looping over it, one
    workgroup per descriptor, two vectors per lane, and the pipelined walk on a fixed grid."""
    import torch
    import kvl_workloads as W
    import paper_2602_21548_amd as K
    dev = torch.device("cuda:0")
    w = W.config(index)
    bs, rows = w.layout.block_tokens, w.layout.row_bytes
    src = [torch.full((w.src.pool_blocks * bs * r,), 3, dtype=torch.uint8, device=dev) for r in rows]
    dst = [torch.full((w.dst.pool_blocks * bs * r,), 0xA5, dtype=torch.uint8, device=dev) for r in rows]
    g = K.kvl_plan(K.make_layout(1, bs, rows, w.src.pool_blocks), w.hit, w.app, w.src.tables, K.KVL_GATHER)
    s = K.kvl_plan(K.make_layout(1, bs, rows, w.dst.pool_blocks), w.hit, w.app, w.dst.tables, K.KVL_SCATTER)
    n = g.payload_bytes
    x = torch.empty(n, dtype=torch.uint8, device=dev)
    stream = torch.cuda.Stream()
    # (name, pack variant, unpack variant): the cache policies are those of the default throughout
    forms = [("default: tiled, one vector per lane", 0, 0),
             ("one wavefront per descriptor, 4 vectors in flight per lane", 22, 30),
             ("one wavefront per descriptor, 8 vectors in flight per lane", 54, 62),
             ("one workgroup per descriptor, 4 vectors in flight per lane", 21, 29),
             ("tiled, two vectors per lane", 24, 32),
             ("pipelined walk on a fixed grid of resident workgroups", 279, 287)]
    out = {"workload": WORKLOADS[index], "unit": "GB/s of memory traffic",
           "note": "every launch is timed alone, the device idle before it and the same kernel run again and again on the same "
                   "buffers: rates for comparing the forms with each other; the rates of the load path itself, with pack and "
                   "unpack alternating and no idle time, are those under other_configs (a few per cent higher)",
           "forms": []}
    for name, vp, vu in forms:
        g.set_tuning(variant=vp)
        s.set_tuning(variant=vu)
        pk = _time_launches(lambda: K.kvl_pack_layer(g, src, x, stream=stream), stream, reps=6)
        up = _time_launches(lambda: K.kvl_unpack_layer(s, x, dst, stream=stream), stream, reps=6)
        out["forms"].append({"form": name, "pack_variant": K.kvl_variant_name(vp), "unpack_variant": K.kvl_variant_name(vu),
                             "pack": round(2.0 * n / pk / 1e6, 1), "unpack": round(2.0 * n / up / 1e6, 1)})
    g.destroy()
    s.destroy()
    del src, dst, x
    torch.cuda.empty_cache()
    return out


def h2d_study(requests: int = 0) -> None:
    """Submission-cost study of the host-buffer load path (Section 5.2 of the paper observes that a
    copy engine fed many small copies is bound by the per-copy submission cost: 5-7 us per copy on
    its hardware).  Prints what the same question looks like here for one layer of the streamed MLA
    workload: one copy per Layer Block, chunked copies through a staging ring at several chunk
    sizes, and the scatter kernel reading the pinned buffer itself."""
    import torch
    import kvl_workloads as W
    import paper_2602_21548_amd as K
    dev = torch.device("cuda:0")
    w = W.config(5, n_requests=requests or None)
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
        for st in streams:
            st.synchronize()
        t2 = time.perf_counter()
        return copies, n / (t2 - t0) / 1e9, (t1 - t0) * 1e6 / max(1, copies)

    best = None
    for _ in range(2):
        best = timed(lambda: K.kvl_h2d_blockwise_layer(plan, host, pool, stream=cs), [cs])
    c, gb, us = best
    print(f"{'one hipMemcpyAsync per Layer Block':44s} {c:8d} {gb:8.2f} {gb / peak:8.1%} {us:16.2f}")
    for mb in (1, 2, 4, 8, 16, 32, 64, 128, 256):
        chunk = mb << 20
        if chunk < bs * max(rows):
            continue
        staging = torch.empty(4 * chunk, dtype=torch.uint8, device=dev)
        copies = len(plan.chunks(chunk))
        res = None
        for _ in range(2):
            res = timed(lambda: (K.kvl_h2d_unpack_layer(plan, host, staging, chunk, pool, cs, ks), copies)[1], [ks, cs])
        c, gb, us = res
        print(f"{'staging ring, chunk ' + str(mb) + ' MiB x 4 slots':44s} {c:8d} {gb:8.2f} {gb / peak:8.1%} {us:16.2f}")
        del staging
    res = None
    for _ in range(2):
        res = timed(lambda: (K.kvl_unpack_layer(plan, host, pool, stream=ks), 1)[1], [ks])
    c, gb, us = res
    print(f"{'scatter kernel reads pinned memory (0 copies)':44s} {0:8d} {gb:8.2f} {gb / peak:8.1%} {us:16.2f}")
    plan.destroy()


if __name__ == "__main__":
    sys.exit(main())
