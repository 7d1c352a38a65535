// Host-buffer paths.  Load: pinned host transfer buffer -> staging slots in HBM
// (hipMemcpyAsync) -> scatter kernel per landed chunk.  The way out mirrors it
// (gather kernel into a slot -> hipMemcpyAsync to the host buffer), and both have
// a form for the storage layout, in which strided copies of the runtime move whole Layer
// Blocks with strided copies and a kernel converts them in HBM.
//
// The paper notes that handing many small copies to a copy engine is bound by
// the per-copy submission cost (Section 5.2), so the host buffer is not copied
// block by block: it is dense, and is cut into multi-megabyte chunks whose ends
// fall on descriptor boundaries; the fine-grained part of the work (finding each
// block's place in the paged pool) is left to the scatter kernel in HBM.
//
// Overlap without per-chunk events: every staging slot has a lane, a stream of the
// library's own, on which that slot's copies and scatters alternate in order
// (copy, scatter, copy, scatter, ...).  In-order execution of a lane keeps a slot
// from being overwritten before it has been scattered; the lanes run side by
// side, so while one lane scatters the others keep the host link busy.  Only the
// layer's start and end touch the caller's streams (a handful of event waits per
// layer).  An earlier form with one copy stream, one kernel stream and two
// events per chunk lost 15-25 % of the link at 8-16 MiB chunks to those events.
#include <dlfcn.h>

#include <algorithm>
#include <new>
#include <vector>

#include "kvl_internal.h"

namespace kvl {

int ensure_lanes(kvl_plan_t *plan, size_t lanes) {
    while (plan->lanes.size() < lanes) {
        hipStream_t s = nullptr;
        if (plan->lane_cu_mask.empty()) {
            s = take_pooled_lane(plan->device);
            if (!s) KVL_HIP(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        } else
            KVL_HIP(hipExtStreamCreateWithCUMask(&s, (uint32_t)plan->lane_cu_mask.size(),
                                                 plan->lane_cu_mask.data()));
        plan->lanes.push_back(s);
    }
    while (plan->ev_lane_done.size() < lanes) {
        hipEvent_t e = nullptr;
        KVL_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        plan->ev_lane_done.push_back(e);
    }
    if (!plan->ev_entry) KVL_HIP(hipEventCreateWithFlags(&plan->ev_entry, hipEventDisableTiming));
    if (!plan->ev_entry2) KVL_HIP(hipEventCreateWithFlags(&plan->ev_entry2, hipEventDisableTiming));
    return KVL_OK;
}

// Order every lane after what the caller has enqueued so far on its two streams.
int lanes_follow(kvl_plan_t *plan, size_t lanes, hipStream_t copy_s, hipStream_t kern_s) {
    KVL_HIP(hipEventRecord(plan->ev_entry, kern_s));
    KVL_HIP(hipEventRecord(plan->ev_entry2, copy_s));
    for (size_t j = 0; j < lanes; ++j) {
        KVL_HIP(hipStreamWaitEvent(plan->lanes[j], plan->ev_entry, 0));
        KVL_HIP(hipStreamWaitEvent(plan->lanes[j], plan->ev_entry2, 0));
    }
    return KVL_OK;
}

// Enqueue one layer on the lanes and make kern_s wait for its end.
// `wait_before_scatter`, if not null, is an event every lane must pass before its
// first scatter of this layer touches the pool (its first copy does not wait).
int enqueue_h2d_layer(kvl_plan_t *plan, const std::vector<kvl_chunk_t> &chunks,
                      const void *host_xfer, void *dev_staging, uint64_t chunk_bytes, size_t lanes,
                      void *const *pool_planes, hipStream_t kern_s, hipEvent_t wait_before_scatter) {
    const char *host = static_cast<const char *>(host_xfer);
    char *stage = static_cast<char *>(dev_staging);
    size_t i = 0;
    for (const kvl_chunk_t &c : chunks) {
        if (c.bytes == 0) continue;
        const size_t lane = i % lanes;
        hipStream_t ls = plan->lanes[lane];
        char *dst = stage + lane * chunk_bytes;
        KVL_HIP(hipMemcpyAsync(dst, host + c.host_offset, c.bytes, hipMemcpyHostToDevice, ls));
        if (i < lanes && wait_before_scatter) KVL_HIP(hipStreamWaitEvent(ls, wait_before_scatter, 0));
        // address at which transfer row 0 of this plane would lie if the whole
        // plane were laid out around this slot
        const uint64_t row = plan->layout.row_bytes[c.plane];
        const uint64_t first_row_off = (uint64_t)plan->units[c.unit_begin].xfer_row * row;
        uintptr_t xp[KVL_MAX_PLANES] = {};
        xp[c.plane] = reinterpret_cast<uintptr_t>(dst) - first_row_off;
        int rc = launch_units(plan, false, c.unit_begin, c.unit_end, c.plane, c.plane + 1,
                              pool_planes, xp, ls);
        if (rc != KVL_OK) return rc;
        ++i;
    }
    const size_t used = std::min(i, lanes);
    for (size_t j = 0; j < used; ++j) {
        KVL_HIP(hipEventRecord(plan->ev_lane_done[j], plan->lanes[j]));
        KVL_HIP(hipStreamWaitEvent(kern_s, plan->ev_lane_done[j], 0));
    }
    return KVL_OK;
}

// Zero-copy form (chunk_bytes == 0): the scatter kernel reads the pinned buffer itself.
int enqueue_zero_copy_layer(const kvl_plan_t *plan, const void *host_xfer, void *const *pool_planes,
                            hipStream_t kern_s, hipEvent_t wait_before_scatter) {
    if (wait_before_scatter) KVL_HIP(hipStreamWaitEvent(kern_s, wait_before_scatter, 0));
    uintptr_t xp[KVL_MAX_PLANES];
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
        xp[p] = reinterpret_cast<uintptr_t>(host_xfer) + plan->plane_base[p];
    return launch_units(plan, false, 0, (uint32_t)plan->units.size(), 0, plan->layout.n_planes,
                        pool_planes, xp, kern_s, is_host_memory(plan, host_xfer));
}

// Staging area of the staged Full-Block load: chunks hold whole Layer Blocks.
int check_fullblock_staging(const kvl_plan_t *plan, const void *staging, uint64_t staging_bytes,
                            uint64_t chunk_bytes, size_t *slots) {
    if (chunk_bytes % 16 || reinterpret_cast<uintptr_t>(staging) % 16) return KVL_EINVAL;
    if (chunk_bytes < layer_block_bytes(plan) || staging_bytes < chunk_bytes) return KVL_ESPACE;
    if (!plan->units.empty() && !staging) return KVL_EINVAL;
    *slots = (size_t)std::min<uint64_t>(staging_bytes / chunk_bytes, 8);
    return KVL_OK;
}

// Per block of a KVL_NO_MERGE plan: its first descriptor and the rows it moves.
// Descriptors of such a plan are in block order and every block has at least one.
static void block_index(kvl_plan_t *plan) {
    const uint64_t nb = plan->blocks_touched;
    if (plan->block_first_unit.size() == nb + 1) return;
    const uint32_t bs = plan->layout.block_tokens;
    plan->block_first_unit.assign(nb + 1, (uint32_t)plan->units.size());
    plan->block_row_lo.assign(nb, bs);
    plan->block_row_hi.assign(nb, 0);
    for (size_t i = plan->units.size(); i-- > 0;) {
        const kvl_unit_t &u = plan->units[i];
        const uint32_t lo = u.pool_row % bs;
        plan->block_first_unit[u.block_index] = (uint32_t)i;
        plan->block_row_lo[u.block_index] = std::min(plan->block_row_lo[u.block_index], lo);
        plan->block_row_hi[u.block_index] = std::max(plan->block_row_hi[u.block_index], lo + u.n_rows);
    }
}

// One layer from a buffer of Full Blocks through the staging slots: per chunk of
// blocks one strided copy (rows of one Layer Block at a pitch of one Full Block)
// and one converting kernel, on the lanes as in enqueue_h2d_layer.
int enqueue_h2d_fullblocks_layer(kvl_plan_t *plan, const void *full_blocks, uint32_t layer,
                                 void *dev_staging, uint64_t chunk_bytes, size_t lanes,
                                 void *const *pool_planes, hipStream_t kern_s, hipEvent_t wait_before_scatter) {
    const uint64_t lb = layer_block_bytes(plan), fb = lb * plan->layout.n_layers;
    const uint64_t nb = plan->blocks_touched, per_chunk = chunk_bytes / lb;
    block_index(plan);
    const char *src = static_cast<const char *>(full_blocks) + (uint64_t)layer * lb;
    char *stage = static_cast<char *>(dev_staging);
    size_t i = 0;
    for (uint64_t b0 = 0; b0 < nb; b0 += per_chunk, ++i) {
        const uint64_t b1 = std::min(nb, b0 + per_chunk);
        const size_t lane = i % lanes;
        hipStream_t ls = plan->lanes[lane];
        char *dst = stage + lane * chunk_bytes;
        KVL_HIP(hipMemcpy2DAsync(dst, lb, src + b0 * fb, fb, lb, b1 - b0, hipMemcpyDefault, ls));
        if (i < lanes && wait_before_scatter) KVL_HIP(hipStreamWaitEvent(ls, wait_before_scatter, 0));
        // block k's Layer Block sits at dst + (k - b0) * lb
        int rc = fullblock_launch(plan, true, reinterpret_cast<uintptr_t>(dst) - b0 * lb, lb, 0,
                                  plan->block_first_unit[b0], plan->block_first_unit[b1], pool_planes, ls);
        if (rc != KVL_OK) return rc;
    }
    const size_t used = std::min(i, lanes);
    for (size_t j = 0; j < used; ++j) {
        KVL_HIP(hipEventRecord(plan->ev_lane_done[j], plan->lanes[j]));
        KVL_HIP(hipStreamWaitEvent(kern_s, plan->ev_lane_done[j], 0));
    }
    return KVL_OK;
}

int check_h2d_args(const kvl_plan_t *plan, const void *host, const void *staging,
                   uint64_t staging_bytes, uint64_t chunk_bytes, size_t *slots) {
    if (!plan) return KVL_EINVAL;
    if (!(plan->flags & KVL_SCATTER) || (plan->flags & KVL_HOST_ONLY)) return KVL_EINVAL;
    if (chunk_bytes == 0) {                 // zero copy: no staging area is needed
        *slots = 0;
        return (!plan->units.empty() && !host) ? KVL_EINVAL : KVL_OK;
    }
    if (chunk_bytes % 16) return KVL_EINVAL;
    if (staging_bytes < chunk_bytes) return KVL_ESPACE;
    if (!plan->units.empty() && (!host || !staging)) return KVL_EINVAL;
    if (reinterpret_cast<uintptr_t>(staging) % 16) return KVL_EINVAL;
    *slots = (size_t)std::min<uint64_t>(staging_bytes / chunk_bytes, 8);    // one lane per slot, at most 8
    return KVL_OK;
}

}  // namespace kvl

static int h2d_unpack_layer(const kvl_plan_t *plan_c, const void *pinned_host_xfer, void *dev_staging,
                            uint64_t staging_bytes, uint64_t chunk_bytes, void *const *pool_planes,
                            void *copy_stream, void *kernel_stream) {
    kvl_plan_t *plan = const_cast<kvl_plan_t *>(plan_c);   // the plan's lanes and events are scratch state
    size_t slots = 0;
    int rc = kvl::check_h2d_args(plan, pinned_host_xfer, dev_staging, staging_bytes, chunk_bytes, &slots);
    if (rc != KVL_OK) return rc;
    if (!pool_planes) return KVL_EINVAL;
    if (plan->units.empty()) return KVL_OK;
    rc = kvl::check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = kvl::check_buffer(plan, pinned_host_xfer, plan->payload_bytes, true);
    if (rc == KVL_OK && chunk_bytes) rc = kvl::check_buffer(plan, dev_staging, slots * chunk_bytes, false);
    if (rc != KVL_OK) return rc;
    if (chunk_bytes == 0)
        return kvl::enqueue_zero_copy_layer(plan, pinned_host_xfer, pool_planes, (hipStream_t)kernel_stream, nullptr);
    std::vector<kvl_chunk_t> chunks;
    rc = kvl::make_chunks(plan, chunk_bytes, chunks);
    if (rc != KVL_OK) return rc;
    rc = kvl::ensure_lanes(plan, slots);
    if (rc != KVL_OK) return rc;
    hipStream_t cs = (hipStream_t)copy_stream, ks = (hipStream_t)kernel_stream;
    rc = kvl::lanes_follow(plan, slots, cs, ks);
    if (rc != KVL_OK) return rc;
    return kvl::enqueue_h2d_layer(plan, chunks, pinned_host_xfer, dev_staging, chunk_bytes, slots,
                                  pool_planes, ks, nullptr);
}

namespace kvl {

// The other direction: gather into the staging slots, copy each landed chunk to
// the pinned host buffer.  On a lane the order is kernel, copy, kernel, copy, ...
// `wait_first`, if not null, is an event every lane passes before its first kernel
// of this layer reads the pool; `collector` is made to wait for the layer's end.
int enqueue_d2h_pack_layer(kvl_plan_t *plan, const std::vector<kvl_chunk_t> &chunks,
                           const void *const *pool_planes, void *dev_staging, uint64_t chunk_bytes,
                           size_t lanes, void *host_xfer, hipEvent_t wait_first, hipStream_t collector) {
    char *host = static_cast<char *>(host_xfer);
    char *stage = static_cast<char *>(dev_staging);
    size_t i = 0;
    for (const kvl_chunk_t &c : chunks) {
        if (c.bytes == 0) continue;
        const size_t lane = i % lanes;
        hipStream_t ls = plan->lanes[lane];
        char *slot = stage + lane * chunk_bytes;
        if (i < lanes && wait_first) KVL_HIP(hipStreamWaitEvent(ls, wait_first, 0));
        const uint64_t first_row_off = (uint64_t)plan->units[c.unit_begin].xfer_row * plan->layout.row_bytes[c.plane];
        uintptr_t xp[KVL_MAX_PLANES] = {};
        xp[c.plane] = reinterpret_cast<uintptr_t>(slot) - first_row_off;
        int rc = launch_units(plan, true, c.unit_begin, c.unit_end, c.plane, c.plane + 1,
                              const_cast<void *const *>(pool_planes), xp, ls);
        if (rc != KVL_OK) return rc;
        KVL_HIP(hipMemcpyAsync(host + c.host_offset, slot, c.bytes, hipMemcpyDeviceToHost, ls));
        ++i;
    }
    const size_t used = std::min(i, lanes);
    for (size_t j = 0; j < used; ++j) {
        KVL_HIP(hipEventRecord(plan->ev_lane_done[j], plan->lanes[j]));
        KVL_HIP(hipStreamWaitEvent(collector, plan->ev_lane_done[j], 0));
    }
    return KVL_OK;
}

// Arguments of a staged gather into host memory; *slots gets the number of lanes.
int check_d2h_args(const kvl_plan_t *plan, const void *staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                   const void *host, uint64_t host_capacity, size_t *slots) {
    if (!plan) return KVL_EINVAL;
    if (!(plan->flags & KVL_GATHER) || (plan->flags & KVL_HOST_ONLY) || plan->paired) return KVL_EINVAL;
    if (chunk_bytes == 0 || chunk_bytes % 16 || reinterpret_cast<uintptr_t>(staging) % 16) return KVL_EINVAL;
    if (staging_bytes < chunk_bytes || host_capacity < plan->payload_bytes) return KVL_ESPACE;
    if (!plan->units.empty() && (!staging || !host)) return KVL_EINVAL;
    *slots = (size_t)std::min<uint64_t>(staging_bytes / chunk_bytes, 8);
    return KVL_OK;
}

}  // namespace kvl

static int d2h_pack_layer(const kvl_plan_t *plan_c, const void *const *pool_planes, void *dev_staging,
                          uint64_t staging_bytes, uint64_t chunk_bytes, void *pinned_host_xfer,
                          uint64_t host_capacity, void *kernel_stream, void *copy_stream) {
    using namespace kvl;
    kvl_plan_t *plan = const_cast<kvl_plan_t *>(plan_c);
    if (!pool_planes) return KVL_EINVAL;
    size_t slots = 0;
    int rc = check_d2h_args(plan, dev_staging, staging_bytes, chunk_bytes, pinned_host_xfer, host_capacity, &slots);
    if (rc != KVL_OK) return rc;
    if (plan->units.empty()) return KVL_OK;
    rc = check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = check_buffer(plan, pinned_host_xfer, plan->payload_bytes, true);
    if (rc == KVL_OK) rc = check_buffer(plan, dev_staging, slots * chunk_bytes, false);
    if (rc != KVL_OK) return rc;
    std::vector<kvl_chunk_t> chunks;
    rc = make_chunks(plan, chunk_bytes, chunks);
    if (rc != KVL_OK) return rc;
    rc = ensure_lanes(plan, slots);
    if (rc != KVL_OK) return rc;
    hipStream_t cs = (hipStream_t)copy_stream, ks = (hipStream_t)kernel_stream;
    rc = lanes_follow(plan, slots, cs, ks);
    if (rc != KVL_OK) return rc;
    return enqueue_d2h_pack_layer(plan, chunks, pool_planes, dev_staging, chunk_bytes, slots, pinned_host_xfer,
                                  nullptr, ks);
}

// Persist direction: one layer of the pool into a buffer of Full Blocks through the
// staging slots.  The kernel lays the blocks' rows out as Layer Blocks in a slot; the
// runtime's copies then write runs of whole blocks with one strided copy each, and the
// rows of partly covered blocks (the ends of a request's range) with one plain copy
// per plane, so that no byte outside the plan's rows is written.
static int d2h_fullblocks_layer(const kvl_plan_t *plan_c, const void *const *pool_planes, uint32_t layer,
                                void *dev_staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                                void *full_blocks, uint64_t full_blocks_bytes, void *kernel_stream,
                                void *copy_stream) {
    using namespace kvl;
    kvl_plan_t *plan = const_cast<kvl_plan_t *>(plan_c);
    if (!pool_planes) return KVL_EINVAL;
    int rc = check_fullblock_args(plan, false, full_blocks_bytes, layer);
    if (rc != KVL_OK) return rc;
    size_t slots = 0;
    rc = check_fullblock_staging(plan, dev_staging, staging_bytes, chunk_bytes, &slots);
    if (rc != KVL_OK) return rc;
    if (plan->units.empty()) return KVL_OK;
    if (!full_blocks) return KVL_EINVAL;
    const uint32_t P = plan->layout.n_planes, bs = plan->layout.block_tokens;
    const uint64_t lb = layer_block_bytes(plan), fb = lb * plan->layout.n_layers;
    const uint64_t nb = plan->blocks_touched, per_chunk = chunk_bytes / lb;
    rc = check_device(plan);
    if (rc == KVL_OK) rc = check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = check_buffer(plan, full_blocks, nb * fb, true);
    if (rc == KVL_OK) rc = check_buffer(plan, dev_staging, slots * chunk_bytes, false);
    if (rc != KVL_OK) return rc;
    rc = ensure_lanes(plan, slots);
    if (rc != KVL_OK) return rc;
    hipStream_t cs = (hipStream_t)copy_stream, ks = (hipStream_t)kernel_stream;
    rc = lanes_follow(plan, slots, cs, ks);
    if (rc != KVL_OK) return rc;
    block_index(plan);
    char *out = static_cast<char *>(full_blocks) + (uint64_t)layer * lb;
    char *stage = static_cast<char *>(dev_staging);
    size_t i = 0;
    for (uint64_t b0 = 0; b0 < nb; b0 += per_chunk, ++i) {
        const uint64_t b1 = std::min(nb, b0 + per_chunk);
        const size_t lane = i % slots;
        hipStream_t ls = plan->lanes[lane];
        char *slot = stage + lane * chunk_bytes;
        rc = fullblock_launch(plan, false, reinterpret_cast<uintptr_t>(slot) - b0 * lb, lb, 0,
                              plan->block_first_unit[b0], plan->block_first_unit[b1],
                              const_cast<void *const *>(pool_planes), ls);
        if (rc != KVL_OK) return rc;
        uint64_t b = b0;
        while (b < b1) {
            const bool whole = plan->block_row_lo[b] == 0 && plan->block_row_hi[b] == bs;
            if (whole) {
                uint64_t e = b + 1;
                while (e < b1 && plan->block_row_lo[e] == 0 && plan->block_row_hi[e] == bs) ++e;
                KVL_HIP(hipMemcpy2DAsync(out + b * fb, fb, slot + (b - b0) * lb, lb, lb, e - b, hipMemcpyDefault, ls));
                b = e;
            } else {
                const uint64_t lo = plan->block_row_lo[b], hi = plan->block_row_hi[b];
                uint64_t plane_off = 0;
                for (uint32_t p = 0; p < P; ++p) {
                    const uint64_t row = plan->layout.row_bytes[p], at = plane_off + lo * row;
                    KVL_HIP(hipMemcpyAsync(out + b * fb + at, slot + (b - b0) * lb + at, (hi - lo) * row,
                                           hipMemcpyDefault, ls));
                    plane_off += (uint64_t)bs * row;
                }
                ++b;
            }
        }
    }
    const size_t used = std::min(i, slots);
    for (size_t j = 0; j < used; ++j) {
        KVL_HIP(hipEventRecord(plan->ev_lane_done[j], plan->lanes[j]));
        KVL_HIP(hipStreamWaitEvent(ks, plan->ev_lane_done[j], 0));
    }
    return KVL_OK;
}

static int h2d_fullblocks_layer(const kvl_plan_t *plan_c, const void *full_blocks, uint64_t full_blocks_bytes,
                                uint32_t layer, void *dev_staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                                void *const *pool_planes, void *copy_stream, void *kernel_stream) {
    using namespace kvl;
    kvl_plan_t *plan = const_cast<kvl_plan_t *>(plan_c);   // lanes, events and the block index are scratch state
    if (!pool_planes) return KVL_EINVAL;
    int rc = check_fullblock_args(plan, true, full_blocks_bytes, layer);
    if (rc != KVL_OK) return rc;
    size_t slots = 0;
    rc = check_fullblock_staging(plan, dev_staging, staging_bytes, chunk_bytes, &slots);
    if (rc != KVL_OK) return rc;
    if (plan->units.empty()) return KVL_OK;
    if (!full_blocks) return KVL_EINVAL;
    const uint64_t fb = layer_block_bytes(plan) * plan->layout.n_layers;
    rc = check_device(plan);
    if (rc == KVL_OK) rc = check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = check_buffer(plan, full_blocks, plan->blocks_touched * fb, true);
    if (rc == KVL_OK) rc = check_buffer(plan, dev_staging, slots * chunk_bytes, false);
    if (rc != KVL_OK) return rc;
    rc = ensure_lanes(plan, slots);
    if (rc != KVL_OK) return rc;
    hipStream_t cs = (hipStream_t)copy_stream, ks = (hipStream_t)kernel_stream;
    rc = lanes_follow(plan, slots, cs, ks);
    if (rc != KVL_OK) return rc;
    return enqueue_h2d_fullblocks_layer(plan, full_blocks, layer, dev_staging, chunk_bytes, slots, pool_planes,
                                        ks, nullptr);
}

extern "C" {

int kvl_h2d_fullblocks_layer(const kvl_plan_t *plan, const void *full_blocks, uint64_t full_blocks_bytes,
                             uint32_t layer, void *dev_staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                             void *const *pool_planes, void *copy_stream, void *kernel_stream) {
    try {
        return h2d_fullblocks_layer(plan, full_blocks, full_blocks_bytes, layer, dev_staging, staging_bytes,
                                    chunk_bytes, pool_planes, copy_stream, kernel_stream);
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
}

int kvl_d2h_fullblocks_layer(const kvl_plan_t *plan, const void *const *pool_planes, uint32_t layer,
                             void *dev_staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                             void *full_blocks, uint64_t full_blocks_bytes, void *kernel_stream,
                             void *copy_stream) {
    try {
        return d2h_fullblocks_layer(plan, pool_planes, layer, dev_staging, staging_bytes, chunk_bytes,
                                    full_blocks, full_blocks_bytes, kernel_stream, copy_stream);
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
}

int kvl_d2h_pack_layer(const kvl_plan_t *plan, const void *const *pool_planes, void *dev_staging,
                       uint64_t staging_bytes, uint64_t chunk_bytes, void *pinned_host_xfer,
                       uint64_t host_capacity, void *kernel_stream, void *copy_stream) {
    try {
        return d2h_pack_layer(plan, pool_planes, dev_staging, staging_bytes, chunk_bytes, pinned_host_xfer,
                              host_capacity, kernel_stream, copy_stream);
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
}

int kvl_h2d_unpack_layer(const kvl_plan_t *plan, const void *pinned_host_xfer, void *dev_staging,
                         uint64_t staging_bytes, uint64_t chunk_bytes, void *const *pool_planes,
                         void *copy_stream, void *kernel_stream) {
    try {
        return h2d_unpack_layer(plan, pinned_host_xfer, dev_staging, staging_bytes, chunk_bytes, pool_planes,
                                copy_stream, kernel_stream);
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
}

int kvl_plan_set_lane_cu_mask(kvl_plan_t *plan, const uint32_t *mask, uint32_t n_words) {
    if (!plan || (n_words && !mask) || (plan->flags & KVL_HOST_ONLY)) return KVL_EINVAL;
    bool any = n_words == 0;
    for (uint32_t i = 0; i < n_words; ++i) any = any || mask[i] != 0;
    if (!any) return KVL_EINVAL;                       // a mask with no compute unit at all
    // the lanes are made anew, under the new mask, by the next call that needs them
    hipError_t first = hipSuccess;
    const bool poolable = plan->lane_cu_mask.empty();       // lanes made without a mask serve any plan
    for (hipStream_t s : plan->lanes) {
        hipError_t e = hipStreamSynchronize(s);
        if (first == hipSuccess) first = e;
        // (the event recorded after the lane's last launch has fired by now and stays with the plan)
        if (poolable) {
            kvl::return_lane(s, plan->device);
        } else {
            e = hipStreamDestroy(s);
            if (first == hipSuccess) first = e;
        }
    }
    plan->lanes.clear();
    try {
        plan->lane_cu_mask.assign(mask, mask + n_words);
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
    if (first != hipSuccess) {
        kvl::set_hip_error(first);
        return KVL_EHIP;
    }
    return KVL_OK;
}

int kvl_h2d_blockwise_layer(const kvl_plan_t *plan, const void *pinned_host_xfer,
                            void *const *pool_planes, void *stream, uint64_t *n_copies) {
    if (!plan || !pool_planes) return KVL_EINVAL;
    if (!(plan->flags & KVL_SCATTER) || (plan->flags & KVL_HOST_ONLY)) return KVL_EINVAL;
    if (n_copies) *n_copies = 0;
    if (plan->units.empty()) return KVL_OK;
    if (!pinned_host_xfer) return KVL_EINVAL;
    int rc = kvl::check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = kvl::check_buffer(plan, pinned_host_xfer, plan->payload_bytes, true);
    if (rc != KVL_OK) return rc;
    const char *host = static_cast<const char *>(pinned_host_xfer);
    uint64_t copies = 0;
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p) {
        if (!pool_planes[p]) return KVL_EINVAL;
        const uint64_t row = plan->layout.row_bytes[p];
        char *pool = static_cast<char *>(pool_planes[p]);
        for (const kvl_unit_t &u : plan->units) {
            KVL_HIP(hipMemcpyAsync(pool + (uint64_t)u.pool_row * row,
                                   host + plan->plane_base[p] + (uint64_t)u.xfer_row * row,
                                   (uint64_t)u.n_rows * row, hipMemcpyHostToDevice, (hipStream_t)stream));
            ++copies;
        }
    }
    if (n_copies) *n_copies = copies;
    return KVL_OK;
}

int kvl_h2d_blockwise_batched_layer(const kvl_plan_t *plan, const void *pinned_host_xfer,
                                    void *const *pool_planes, void *stream, uint64_t *n_copies) {
    // looked up at run time: the library also has to load under runtimes that predate the call
    typedef hipError_t (*batch_fn)(void **, void **, size_t *, size_t, void *, size_t *, size_t, size_t *, hipStream_t);
    static const batch_fn batch = reinterpret_cast<batch_fn>(dlsym(RTLD_DEFAULT, "hipMemcpyBatchAsync"));
    if (!plan || !pool_planes) return KVL_EINVAL;
    if (!(plan->flags & KVL_SCATTER) || (plan->flags & KVL_HOST_ONLY)) return KVL_EINVAL;
    if (n_copies) *n_copies = 0;
    if (!batch) return KVL_ENOSYS;
    if (plan->units.empty()) return KVL_OK;
    if (!pinned_host_xfer) return KVL_EINVAL;
    int rc = kvl::check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = kvl::check_buffer(plan, pinned_host_xfer, plan->payload_bytes, true);
    if (rc != KVL_OK) return rc;
    try {
        const size_t n = plan->units.size() * plan->layout.n_planes;
        std::vector<void *> dsts(n), srcs(n);
        std::vector<size_t> sizes(n);
        char *host = static_cast<char *>(const_cast<void *>(pinned_host_xfer));
        size_t k = 0;
        for (uint32_t p = 0; p < plan->layout.n_planes; ++p) {
            const uint64_t row = plan->layout.row_bytes[p];
            char *pool = static_cast<char *>(pool_planes[p]);
            for (const kvl_unit_t &u : plan->units) {
                dsts[k] = pool + (uint64_t)u.pool_row * row;
                srcs[k] = host + plan->plane_base[p] + (uint64_t)u.xfer_row * row;
                sizes[k] = (size_t)u.n_rows * row;
                ++k;
            }
        }
        size_t fail = 0;
        KVL_HIP(batch(dsts.data(), srcs.data(), sizes.data(), n, nullptr, nullptr, 0, &fail, (hipStream_t)stream));
        if (n_copies) *n_copies = n;
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
    return KVL_OK;
}

int kvl_measure_h2d_peak(const void *pinned_host, void *dev, uint64_t bytes, uint32_t reps,
                         void *stream, double *gbps) {
    if (!pinned_host || !dev || !gbps || bytes == 0 || reps == 0) return KVL_EINVAL;
    int rc = kvl_check_buffer(pinned_host, bytes, 1);
    if (rc == KVL_OK) rc = kvl_check_buffer(dev, bytes, 0);
    if (rc != KVL_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t a = nullptr, b = nullptr;
    KVL_HIP(hipEventCreate(&a));
    hipError_t e = hipEventCreate(&b);
    if (e != hipSuccess) { (void)hipEventDestroy(a); kvl::set_hip_error(e); return KVL_EHIP; }
    double best = 0.0;
    for (uint32_t i = 0; i < reps && e == hipSuccess; ++i) {
        e = hipEventRecord(a, s);
        if (e == hipSuccess) e = hipMemcpyAsync(dev, pinned_host, bytes, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipEventRecord(b, s);
        if (e == hipSuccess) e = hipEventSynchronize(b);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, b);
        if (e == hipSuccess && ms > 0.f) best = std::max(best, (double)bytes / (ms * 1e-3) / 1e9);
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (e != hipSuccess) { kvl::set_hip_error(e); return KVL_EHIP; }
    *gbps = best;
    return KVL_OK;
}

}  // extern "C"
