// Layer-wise streamed load: the host-buffer load of layer l+1 runs under the
// compute of layer l (Section 4.1: transfers overlap the forward pass; with
// layer-wise prefill only a few layers' cache is resident at a time).
//
// Three streams and a handful of events carry the ordering:
//   lanes          (library-owned, one per staging slot) host -> staging copy and
//                  scatter of each chunk, alternating in order; a lane's first
//                  scatter of layer l waits for "compute of layer l - S finished"
//                  (the slot it is about to overwrite is no longer being read)
//   kernel stream  collects the lanes at the end of each layer: "layer l loaded"
//   compute stream compute(l) waits for "layer l loaded"
#include <algorithm>
#include <new>
#include <vector>

#include "kvl_internal.h"

namespace kvl {

typedef uint32_t v4u __attribute__((ext_vector_type(4)));

struct SlotPlanes {
    uintptr_t base[KVL_MAX_PLANES];
};

// Stand-in for one layer's forward computation: samples what it can see of the
// loaded cache, then holds the compute stream for a fixed time on the device's
// constant-rate wall clock.  One wavefront; the spin ends on the clock or, as a
// backstop, after max_polls polls.
__global__ void __launch_bounds__(64) kvl_compute_kernel(SlotPlanes slot, const kvl_probe_t *probes,
                                                         uint32_t n_probes, v4u *probe_out,
                                                         uint64_t ticks, uint32_t max_polls) {
    for (uint32_t i = threadIdx.x; i < n_probes; i += blockDim.x) {
        const kvl_probe_t pr = probes[i];
        probe_out[i] = *reinterpret_cast<const v4u *>(slot.base[pr.plane] + pr.byte_offset);
    }
    if (threadIdx.x == 0) {
        const uint64_t t0 = wall_clock64();
        for (uint32_t k = 0; k < max_polls; ++k) {
            if (wall_clock64() - t0 >= ticks) break;
            __builtin_amdgcn_s_sleep(8);
        }
    }
}

struct RunState {
    std::vector<hipEvent_t> events;
    kvl_probe_t *d_probes = nullptr;
    hipStream_t streams[3] = {nullptr, nullptr, nullptr};
    const std::vector<hipStream_t> *lanes = nullptr;
    const std::vector<hipStream_t> *out_lanes = nullptr;

    int make(hipEvent_t *e, bool timing) {
        KVL_HIP(hipEventCreateWithFlags(e, timing ? hipEventDefault : hipEventDisableTiming));
        events.push_back(*e);
        return KVL_OK;
    }
    ~RunState() {
        // nothing enqueued by the run may outlive what it refers to
        if (lanes)
            for (hipStream_t s : *lanes) (void)hipStreamSynchronize(s);
        if (out_lanes)
            for (hipStream_t s : *out_lanes) (void)hipStreamSynchronize(s);
        for (hipStream_t s : streams) (void)hipStreamSynchronize(s);
        for (hipEvent_t e : events) (void)hipEventDestroy(e);
        if (d_probes) (void)hipFree(d_probes);
    }
};

}  // namespace kvl

static int stream_layers(const kvl_plan_t *plan_c, const kvl_stream_cfg_t *cfg, kvl_stream_stats_t *stats) {
    using namespace kvl;
    kvl_plan_t *plan = const_cast<kvl_plan_t *>(plan_c);
    if (!plan || !cfg) return KVL_EINVAL;
    const uint32_t L = cfg->n_layers ? cfg->n_layers : plan->layout.n_layers;
    const uint32_t H = cfg->n_host_slots, S = cfg->n_dev_slots, P = plan->layout.n_planes;
    const bool from_blocks = cfg->full_blocks != nullptr;
    if (L == 0 || S == 0 || !cfg->dev_slot_planes) return KVL_EINVAL;
    if (!from_blocks && (H == 0 || !cfg->host_layers)) return KVL_EINVAL;
    if (cfg->compute_us > 1000000u) return KVL_EINVAL;
    if (cfg->n_probes && (!cfg->probes || !cfg->probe_out)) return KVL_EINVAL;
    if (cfg->compute && cfg->n_probes) return KVL_EINVAL;     // the probes belong to the synthetic kernel
    size_t slots = 0;
    int rc = KVL_OK;
    if (from_blocks) {
        if (!(plan->flags & KVL_SCATTER) || (plan->flags & KVL_HOST_ONLY) || !(plan->flags & KVL_NO_MERGE))
            return KVL_EINVAL;
        if (L > plan->layout.n_layers) return KVL_EINVAL;
        rc = check_fullblock_args(plan, true, cfg->full_blocks_bytes, L - 1);
        if (rc != KVL_OK) return rc;
        if (cfg->chunk_bytes) {         // staged form: strided copies bring the Layer Blocks in
            rc = check_fullblock_staging(plan, cfg->dev_staging, cfg->staging_bytes, cfg->chunk_bytes, &slots);
            if (rc != KVL_OK) return rc;
        }
    } else {
        rc = check_h2d_args(plan, cfg->host_layers[0], cfg->dev_staging, cfg->staging_bytes,
                            cfg->chunk_bytes, &slots);
        if (rc != KVL_OK) return rc;
        for (uint32_t h = 0; h < H; ++h)
            if (!cfg->host_layers[h] && !plan->units.empty()) return KVL_EINVAL;
    }
    for (uint32_t i = 0; i < S * P; ++i)
        if (!cfg->dev_slot_planes[i]) return KVL_EINVAL;
    if (!plan->units.empty()) {
        for (uint32_t sl = 0; sl < S && rc == KVL_OK; ++sl)
            rc = check_pool(plan, cfg->dev_slot_planes + (size_t)sl * P, plan->layout.pool_blocks);
        if (!from_blocks) {
            for (uint32_t h = 0; h < H && rc == KVL_OK; ++h)
                rc = check_buffer(plan, cfg->host_layers[h], plan->payload_bytes, true);
        }
        if (rc == KVL_OK && cfg->chunk_bytes)
            rc = check_buffer(plan, cfg->dev_staging, slots * cfg->chunk_bytes, false);
        if (rc != KVL_OK) return rc;
    }
    if (cfg->n_probes) {
        rc = check_buffer(plan, cfg->probe_out, (uint64_t)L * cfg->n_probes * 16, false);
        if (rc != KVL_OK) return rc;
    }
    if (cfg->snapshot_planes) {
        for (size_t i = 0; i < (size_t)L * P; ++i) {
            if (!cfg->snapshot_planes[i]) continue;
            const uint64_t bytes = plan->layout.pool_blocks * plan->layout.block_tokens *
                                   (uint64_t)plan->layout.row_bytes[i % P];
            rc = check_buffer(plan, cfg->snapshot_planes[i], bytes, false);
            if (rc != KVL_OK) return rc;
        }
    }
    for (uint32_t i = 0; i < cfg->n_probes; ++i) {
        const kvl_probe_t &pr = cfg->probes[i];
        const uint64_t plane_bytes = plan->layout.pool_blocks * plan->layout.block_tokens *
                                     (uint64_t)plan->layout.row_bytes[pr.plane < P ? pr.plane : 0];
        if (pr.plane >= P || pr.byte_offset % 16 || pr.byte_offset + 16 > plane_bytes) return KVL_EINVAL;
    }

    // outflow
    kvl_plan_t *oplan = const_cast<kvl_plan_t *>(cfg->out_plan);
    const uint32_t Ho = cfg->n_out_host_slots;
    size_t oslots = 0;
    std::vector<kvl_chunk_t> ochunks;
    if (oplan) {
        if (oplan == plan || Ho == 0 || !cfg->out_host_layers) return KVL_EINVAL;
        if (!(oplan->flags & KVL_GATHER) || (oplan->flags & KVL_HOST_ONLY) || oplan->paired) return KVL_EINVAL;
        const kvl_layout_t &a = plan->layout, &b = oplan->layout;
        if (a.block_tokens != b.block_tokens || a.n_planes != b.n_planes || a.pool_blocks != b.pool_blocks ||
            oplan->device != plan->device)
            return KVL_EINVAL;
        for (uint32_t p = 0; p < P; ++p)
            if (a.row_bytes[p] != b.row_bytes[p]) return KVL_EINVAL;
        for (uint32_t h = 0; h < Ho; ++h) {
            if (!cfg->out_host_layers[h] && !oplan->units.empty()) return KVL_EINVAL;
            if (!oplan->units.empty()) {
                rc = check_buffer(oplan, cfg->out_host_layers[h], oplan->payload_bytes, true);
                if (rc != KVL_OK) return rc;
            }
        }
        if (cfg->out_chunk_bytes) {
            rc = check_d2h_args(oplan, cfg->out_staging, cfg->out_staging_bytes, cfg->out_chunk_bytes,
                                cfg->out_host_layers[0], oplan->payload_bytes, &oslots);
            if (rc == KVL_OK && !oplan->units.empty())
                rc = check_buffer(oplan, cfg->out_staging, oslots * cfg->out_chunk_bytes, false);
            if (rc == KVL_OK) rc = make_chunks(oplan, cfg->out_chunk_bytes, ochunks);
            if (rc != KVL_OK) return rc;
        }
        rc = ensure_lanes(oplan, oslots ? oslots : 1);
        if (rc != KVL_OK) return rc;
    }

    std::vector<kvl_chunk_t> chunks;
    const bool zero_copy = !from_blocks && cfg->chunk_bytes == 0;
    if (!from_blocks && !zero_copy) {
        rc = make_chunks(plan, cfg->chunk_bytes, chunks);
        if (rc != KVL_OK) return rc;
    }
    rc = ensure_lanes(plan, slots ? slots : 1);
    if (rc != KVL_OK) return rc;

    hipStream_t cs = (hipStream_t)cfg->copy_stream, ks = (hipStream_t)cfg->kernel_stream,
                ms = (hipStream_t)cfg->compute_stream;
    int clock_khz = 0;
    KVL_HIP(hipDeviceGetAttribute(&clock_khz, hipDeviceAttributeWallClockRate, plan->device));
    if (clock_khz <= 0) clock_khz = 100000;
    const uint64_t ticks = (uint64_t)cfg->compute_us * (uint64_t)clock_khz / 1000u;
    // each poll sleeps a fraction of a microsecond; this bound is far beyond compute_us
    const uint32_t max_polls = cfg->compute_us * 64u + 1024u;

    RunState st;
    st.streams[0] = cs; st.streams[1] = ks; st.streams[2] = ms;
    st.lanes = &plan->lanes;
    if (oplan) st.out_lanes = &oplan->lanes;
    hipEvent_t ev_start = nullptr, ev_sync = nullptr;
    std::vector<hipEvent_t> loaded(L), cbeg(L), cend(L), h2d_done(L), out_done(oplan ? L : 0);
    st.events.reserve(5 * (size_t)L + 2);
    if ((rc = st.make(&ev_start, true)) != KVL_OK) return rc;
    if ((rc = st.make(&ev_sync, false)) != KVL_OK) return rc;
    for (uint32_t l = 0; l < L; ++l) {
        if ((rc = st.make(&loaded[l], true)) != KVL_OK) return rc;
        if ((rc = st.make(&cbeg[l], true)) != KVL_OK) return rc;
        if ((rc = st.make(&cend[l], true)) != KVL_OK) return rc;
        if ((rc = st.make(&h2d_done[l], false)) != KVL_OK) return rc;
        if (oplan && (rc = st.make(&out_done[l], true)) != KVL_OK) return rc;
    }
    if (cfg->n_probes) {
        const size_t bytes = cfg->n_probes * sizeof(kvl_probe_t);
        KVL_HIP(hipMalloc((void **)&st.d_probes, bytes));
        KVL_HIP(hipMemcpy(st.d_probes, cfg->probes, bytes, hipMemcpyHostToDevice));
    }

    // start line: the copy stream begins after whatever the other two hold
    KVL_HIP(hipEventRecord(ev_sync, ks));
    KVL_HIP(hipStreamWaitEvent(cs, ev_sync, 0));
    KVL_HIP(hipEventRecord(plan->ev_entry, ms));
    KVL_HIP(hipStreamWaitEvent(cs, plan->ev_entry, 0));
    KVL_HIP(hipEventRecord(ev_start, cs));
    KVL_HIP(hipStreamWaitEvent(ks, ev_start, 0));
    KVL_HIP(hipStreamWaitEvent(ms, ev_start, 0));

    // the lanes start where the three streams start
    const bool staged_blocks = from_blocks && cfg->chunk_bytes != 0;
    if ((!from_blocks && !zero_copy) || staged_blocks) {
        rc = lanes_follow(plan, slots, cs, ks);
        if (rc != KVL_OK) return rc;
    }
    for (uint32_t l = 0; l < L; ++l) {
        const uint32_t s = l % S;
        void *const *slot_planes = cfg->dev_slot_planes + (size_t)s * P;
        // the slot may be overwritten once what read it last has finished: the compute of
        // layer l - S, or, with an outflow, that layer's gather
        hipEvent_t slot_free = l >= S ? (oplan ? out_done[l - S] : cend[l - S]) : nullptr;
        if (staged_blocks) {
            rc = plan->units.empty() ? KVL_OK
                                     : enqueue_h2d_fullblocks_layer(plan, cfg->full_blocks, l, cfg->dev_staging,
                                                                    cfg->chunk_bytes, slots, slot_planes, ks,
                                                                    slot_free);
        } else if (from_blocks) {
            // the slot may be overwritten once the compute that read it has finished
            if (slot_free) KVL_HIP(hipStreamWaitEvent(ks, slot_free, 0));
            rc = fullblock_layer(plan, true, reinterpret_cast<uintptr_t>(cfg->full_blocks),
                                 cfg->full_blocks_bytes, l, slot_planes, ks);
        } else {
            void *host_slot = cfg->host_layers[l % H];
            if (cfg->host_fill) {
                if (l >= H) KVL_HIP(hipEventSynchronize(h2d_done[l - H]));
                if (cfg->host_fill(cfg->host_fill_user, l, host_slot, plan->payload_bytes) != 0)
                    return KVL_EINVAL;
            }
            if (zero_copy) {
                rc = plan->units.empty() ? KVL_OK
                                         : enqueue_zero_copy_layer(plan, host_slot, slot_planes, ks,
                                                                   slot_free);
                // the host slot is free again once this kernel has read it
                if (rc == KVL_OK) KVL_HIP(hipEventRecord(h2d_done[l], ks));
            } else {
                rc = enqueue_h2d_layer(plan, chunks, host_slot, cfg->dev_staging, cfg->chunk_bytes, slots,
                                       slot_planes, ks, slot_free);
                // every copy of the layer has been scattered by then: the host slot is free again
                if (rc == KVL_OK) KVL_HIP(hipEventRecord(h2d_done[l], ks));
            }
        }
        if (rc != KVL_OK) return rc;
        KVL_HIP(hipEventRecord(loaded[l], ks));

        KVL_HIP(hipStreamWaitEvent(ms, loaded[l], 0));
        KVL_HIP(hipEventRecord(cbeg[l], ms));
        SlotPlanes sp{};
        for (uint32_t p = 0; p < P; ++p) sp.base[p] = reinterpret_cast<uintptr_t>(slot_planes[p]);
        v4u *pout = cfg->n_probes
                        ? static_cast<v4u *>(cfg->probe_out) + (size_t)l * cfg->n_probes
                        : nullptr;
        if (cfg->compute) {
            if (cfg->compute(cfg->compute_user, l, slot_planes, cfg->compute_stream) != 0) return KVL_EINVAL;
        } else {
            hipLaunchKernelGGL(kvl_compute_kernel, dim3(1), dim3(64), 0, ms, sp, st.d_probes,
                               cfg->n_probes, pout, ticks, max_polls);
            KVL_HIP(hipGetLastError());
        }
        if (cfg->snapshot_planes) {
            for (uint32_t p = 0; p < P; ++p) {
                void *snap = cfg->snapshot_planes[(size_t)l * P + p];
                if (!snap) continue;
                const uint64_t bytes = plan->layout.pool_blocks * plan->layout.block_tokens *
                                       (uint64_t)plan->layout.row_bytes[p];
                KVL_HIP(hipMemcpyAsync(snap, slot_planes[p], bytes, hipMemcpyDeviceToDevice, ms));
            }
        }
        KVL_HIP(hipEventRecord(cend[l], ms));

        if (oplan) {
            void *out_host = cfg->out_host_layers[l % Ho];
            if (l >= Ho) {          // the buffer still holds layer l - Ho: let the caller have it first
                KVL_HIP(hipEventSynchronize(out_done[l - Ho]));
                if (cfg->host_drain &&
                    cfg->host_drain(cfg->host_drain_user, l - Ho, out_host, oplan->payload_bytes) != 0)
                    return KVL_EINVAL;
            }
            if (oplan->units.empty()) {
                KVL_HIP(hipStreamWaitEvent(cs, cend[l], 0));
            } else if (cfg->out_chunk_bytes) {
                rc = enqueue_d2h_pack_layer(oplan, ochunks, const_cast<const void *const *>(slot_planes),
                                            cfg->out_staging, cfg->out_chunk_bytes, oslots, out_host, cend[l], cs);
                if (rc != KVL_OK) return rc;
            } else {                // the gather writes the host buffer itself
                KVL_HIP(hipStreamWaitEvent(cs, cend[l], 0));
                uintptr_t xp[KVL_MAX_PLANES];
                for (uint32_t p = 0; p < P; ++p)
                    xp[p] = reinterpret_cast<uintptr_t>(out_host) + oplan->plane_base[p];
                rc = launch_units(oplan, true, 0, (uint32_t)oplan->units.size(), 0, P, slot_planes, xp, cs,
                                  is_host_memory(oplan, out_host));
                if (rc != KVL_OK) return rc;
            }
            KVL_HIP(hipEventRecord(out_done[l], cs));
        }
    }
    KVL_HIP(hipEventSynchronize(cend[L - 1]));
    if (oplan) {
        for (uint32_t l = L > Ho ? L - Ho : 0; l < L; ++l) {
            KVL_HIP(hipEventSynchronize(out_done[l]));
            if (cfg->host_drain &&
                cfg->host_drain(cfg->host_drain_user, l, cfg->out_host_layers[l % Ho], oplan->payload_bytes) != 0)
                return KVL_EINVAL;
        }
    }
    KVL_HIP(hipStreamSynchronize(ks));
    KVL_HIP(hipStreamSynchronize(cs));

    if (stats) {
        float total = 0.f;
        KVL_HIP(hipEventElapsedTime(&total, ev_start, cend[L - 1]));
        if (oplan) {
            float t = 0.f;
            KVL_HIP(hipEventElapsedTime(&t, ev_start, out_done[L - 1]));
            total = std::max(total, t);
        }
        stats->d2h_bytes = oplan ? (double)oplan->payload_bytes * L : 0.0;
        stats->out_gbps = (oplan && total > 0.f) ? stats->d2h_bytes / (total * 1e-3) / 1e9 : 0.0;
        stats->total_ms = total;
        stats->h2d_bytes = (double)plan->payload_bytes * L;
        stats->link_gbps = total > 0.f ? stats->h2d_bytes / (total * 1e-3) / 1e9 : 0.0;
        double computed = (double)L * cfg->compute_us * 1e-3;
        if (cfg->compute) {
            computed = 0.0;
            for (uint32_t l = 0; l < L; ++l) {
                float t = 0.f;
                KVL_HIP(hipEventElapsedTime(&t, cbeg[l], cend[l]));
                computed += t;
            }
        }
        stats->exposed_ms = total - computed;
        for (uint32_t l = 0; l < L; ++l) {
            float t = 0.f;
            if (stats->t_loaded) {
                KVL_HIP(hipEventElapsedTime(&t, ev_start, loaded[l]));
                stats->t_loaded[l] = t;
            }
            if (stats->t_compute_begin) {
                KVL_HIP(hipEventElapsedTime(&t, ev_start, cbeg[l]));
                stats->t_compute_begin[l] = t;
            }
            if (stats->t_compute_end) {
                KVL_HIP(hipEventElapsedTime(&t, ev_start, cend[l]));
                stats->t_compute_end[l] = t;
            }
            if (stats->t_out_done && oplan) {
                KVL_HIP(hipEventElapsedTime(&t, ev_start, out_done[l]));
                stats->t_out_done[l] = t;
            }
        }
    }
    return KVL_OK;
}

extern "C" int kvl_stream_layers(const kvl_plan_t *plan, const kvl_stream_cfg_t *cfg, kvl_stream_stats_t *stats) {
    try {
        return stream_layers(plan, cfg, stats);
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
}
