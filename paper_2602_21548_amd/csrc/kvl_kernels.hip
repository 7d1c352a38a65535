// Launchers of the copy kernels and the entry points built on them (pack, unpack, move,
// storage layout, plain copy).  The kernels themselves are in kvl_copy_kernels.h.
#include <algorithm>
#include <cstdio>

#include "kvl_copy_kernels.h"

namespace kvl {

// Every plane of a pool must be device-addressable memory of the pool's full size.
int check_pool(const kvl_plan_t *plan, const void *const *planes, uint64_t pool_blocks) {
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p) {
        if (!planes[p]) return KVL_EINVAL;
        const uint64_t bytes = pool_blocks * plan->layout.block_tokens * (uint64_t)plan->layout.row_bytes[p];
        int rc = check_buffer(plan, planes[p], bytes, false);
        if (rc != KVL_OK) return rc;
    }
    return KVL_OK;
}

// The descriptors live on the device that was current when the plan was made.
int check_device(const kvl_plan_t *plan) {
    int dev = -1;
    KVL_HIP(hipGetDevice(&dev));
    return dev == plan->device ? KVL_OK : KVL_EINVAL;
}

template <bool PACK, bool WAVE, int U, bool NTL, int SP>
static void launch_one(dim3 grid, dim3 block, hipStream_t s, const CopyArgs &a) {
    if (PACK) hipLaunchKernelGGL((kvl_pack_kernel<WAVE, U, NTL, SP>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((kvl_unpack_kernel<WAVE, U, NTL, SP>), grid, block, 0, s, a);
}

template <bool PACK, bool WAVE, int U, bool NTL>
static void launch_sp(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a) {
    switch ((v >> 3) & 3u) {
        case 0: launch_one<PACK, WAVE, U, NTL, 0>(g, b, s, a); break;
        case 1: launch_one<PACK, WAVE, U, NTL, 1>(g, b, s, a); break;
        case 2: launch_one<PACK, WAVE, U, NTL, 2>(g, b, s, a); break;
        default: launch_one<PACK, WAVE, U, NTL, 3>(g, b, s, a); break;
    }
}

template <bool PACK, bool WAVE, int U>
static void launch_nt(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a) {
    if (v & 4u) launch_sp<PACK, WAVE, U, true>(v, g, b, s, a);
    else launch_sp<PACK, WAVE, U, false>(v, g, b, s, a);
}

template <bool PACK>
static void launch_span_variant(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a) {
    const bool wave = (v & 3u) == 1u, deep = (v & 32u) != 0;
    if (wave) {
        if (deep) launch_nt<PACK, true, 8>(v, g, b, s, a);
        else launch_nt<PACK, true, 4>(v, g, b, s, a);
    } else {
        if (deep) launch_nt<PACK, false, 8>(v, g, b, s, a);
        else launch_nt<PACK, false, 4>(v, g, b, s, a);
    }
}

// n_tiles != 0: the launch has fewer workgroups than tiles and they walk over them
template <bool PACK, int VPT, bool NTL, int SP>
static void launch_tile_one(dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu, uint32_t al,
                            uint32_t n_tiles) {
    if (n_tiles) hipLaunchKernelGGL((kvl_tile_walk_kernel<PACK, VPT, NTL, SP>), g, b, 0, s, a, tpu, al, n_tiles);
    else if (PACK) hipLaunchKernelGGL((kvl_pack_tile_kernel<VPT, NTL, SP>), g, b, 0, s, a, tpu, al);
    else hipLaunchKernelGGL((kvl_unpack_tile_kernel<VPT, NTL, SP>), g, b, 0, s, a, tpu, al);
}

template <bool PACK, int VPT, bool NTL>
static void launch_tile_sp(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu,
                           uint32_t al, uint32_t n_tiles) {
    switch ((v >> 3) & 3u) {
        case 0: launch_tile_one<PACK, VPT, NTL, 0>(g, b, s, a, tpu, al, n_tiles); break;
        case 1: launch_tile_one<PACK, VPT, NTL, 1>(g, b, s, a, tpu, al, n_tiles); break;
        case 2: launch_tile_one<PACK, VPT, NTL, 2>(g, b, s, a, tpu, al, n_tiles); break;
        default: launch_tile_one<PACK, VPT, NTL, 3>(g, b, s, a, tpu, al, n_tiles); break;
    }
}

template <bool PACK, int VPT>
static void launch_tile_variant(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu,
                                uint32_t al, uint32_t n_tiles) {
    if (v & 4u) launch_tile_sp<PACK, VPT, true>(v, g, b, s, a, tpu, al, n_tiles);
    else launch_tile_sp<PACK, VPT, false>(v, g, b, s, a, tpu, al, n_tiles);
}

template <bool PACK, bool NTL>
static void launch_pipe_sp(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu, uint32_t al,
                           uint32_t n_tiles) {
    switch ((v >> 3) & 3u) {
        case 0: hipLaunchKernelGGL((kvl_tile_pipe_kernel<PACK, NTL, 0>), g, b, 0, s, a, tpu, al, n_tiles); break;
        case 1: hipLaunchKernelGGL((kvl_tile_pipe_kernel<PACK, NTL, 1>), g, b, 0, s, a, tpu, al, n_tiles); break;
        case 2: hipLaunchKernelGGL((kvl_tile_pipe_kernel<PACK, NTL, 2>), g, b, 0, s, a, tpu, al, n_tiles); break;
        default: hipLaunchKernelGGL((kvl_tile_pipe_kernel<PACK, NTL, 3>), g, b, 0, s, a, tpu, al, n_tiles); break;
    }
}

template <bool PACK>
static void launch_pipe_variant(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu,
                                uint32_t al, uint32_t n_tiles) {
    if (v & 4u) launch_pipe_sp<PACK, true>(v, g, b, s, a, tpu, al, n_tiles);
    else launch_pipe_sp<PACK, false>(v, g, b, s, a, tpu, al, n_tiles);
}

// Compute units of a device (asked once per device).
static int compute_units(int device) {
    static int cached[64] = {};
    if (device < 0 || device >= 64) return 256;
    if (cached[device] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n <= 0) {
            (void)hipGetLastError();
            n = 256;
        }
        cached[device] = n;
    }
    return cached[device];
}

template <bool PACK, bool NTL>
static void launch_flat_sp(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t mur) {
    switch ((v >> 3) & 3u) {
        case 0: hipLaunchKernelGGL((kvl_flat_kernel<PACK, NTL, 0>), g, b, 0, s, a, mur); break;
        case 1: hipLaunchKernelGGL((kvl_flat_kernel<PACK, NTL, 1>), g, b, 0, s, a, mur); break;
        case 2: hipLaunchKernelGGL((kvl_flat_kernel<PACK, NTL, 2>), g, b, 0, s, a, mur); break;
        default: hipLaunchKernelGGL((kvl_flat_kernel<PACK, NTL, 3>), g, b, 0, s, a, mur); break;
    }
}

template <bool PACK>
static void launch_flat_variant(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t mur) {
    if (v & 4u) launch_flat_sp<PACK, true>(v, g, b, s, a, mur);
    else launch_flat_sp<PACK, false>(v, g, b, s, a, mur);
}

int launch_units(const kvl_plan_t *plan, bool pack, uint32_t unit_begin, uint32_t unit_end,
                 uint32_t plane_begin, uint32_t plane_end,
                 void *const *pool_planes, const uintptr_t *xfer_plane, hipStream_t stream, bool far_host) {
    if (unit_end <= unit_begin || plane_end <= plane_begin) return KVL_OK;
    if (!plan->d_units || unit_end > plan->units.size() || plane_end > plan->layout.n_planes)
        return KVL_EINVAL;
    // Planes of different row sizes go in launches of their own: one launch gives every plane the
    // tile count of the widest, and a narrow plane's workgroups would mostly find nothing to do
    // (K/V-style planes of 1024 and 128 bytes in one launch: 2.8 TB/s; apart: 6 TB/s and more).
    for (uint32_t p = plane_begin + 1; p < plane_end; ++p) {
        if (plan->layout.row_bytes[p] == plan->layout.row_bytes[plane_begin]) continue;
        for (uint32_t q = plane_begin; q < plane_end;) {
            uint32_t e = q + 1;
            while (e < plane_end && plan->layout.row_bytes[e] == plan->layout.row_bytes[q]) ++e;
            int rc = launch_units(plan, pack, unit_begin, unit_end, q, e, pool_planes, xfer_plane, stream, far_host);
            if (rc != KVL_OK) return rc;
            q = e;
        }
        return KVL_OK;
    }
    int rc_dev = check_device(plan);
    if (rc_dev != KVL_OK) return rc_dev;
    CopyArgs a{};
    a.units = plan->d_units;
    a.unit_begin = unit_begin;
    a.n_units = unit_end - unit_begin;
    a.plane_begin = plane_begin;
    bool vec = plan->vec16;
    for (uint32_t p = plane_begin; p < plane_end; ++p) {
        if (!pool_planes[p]) return KVL_EINVAL;
        a.pool[p] = reinterpret_cast<uintptr_t>(pool_planes[p]);
        a.xfer[p] = xfer_plane[p];
        vec = vec && (a.pool[p] % 16 == 0) && (a.xfer[p] % 16 == 0);
    }
    for (uint32_t p = plane_begin; p < plane_end; ++p)
        a.row_elems[p] = vec ? plan->layout.row_bytes[p] / 16 : plan->layout.row_bytes[p];

    uint32_t threads = plan->tuning.block_threads;
    // default: tiled, one vector per lane; cache policies as measured (see the top of kvl_copy_kernels.h)
    uint32_t v;
    if (plan->tuning.variant) {
        v = plan->tuning.variant - 1;
    } else {
        bool rows_128 = true;       // every span starts on a 128-byte line of the transfer buffer
        for (uint32_t p = plane_begin; p < plane_end; ++p)
            rows_128 = rows_128 && plan->layout.row_bytes[p] % 128 == 0;
        if (pack) v = kDefaultPackCode;
        else v = rows_128 ? kDefaultUnpackCode : kDefaultUnpackCodeOddRows;
        // across the host link: two vectors per lane, so that the few workgroups of the thin
        // form (kHostSideGroups) keep enough bytes in flight
        if (far_host) v |= 3u;
    }
    if (v & 256u) v = (v & ~(3u | 32u | 128u)) | 2u;      // the pipelined form is a tiled one, one vector per lane
    uint32_t widest = 0;        // vectors of the largest descriptor, over the planes of this launch
    for (uint32_t p = plane_begin; p < plane_end; ++p) widest = std::max(widest, a.row_elems[p]);
    const uint64_t unit_vecs = (uint64_t)plan->max_unit_rows * widest;
    // Descriptors that fill their last tile badly: with the default workgroup size, halve it where that
    // leaves clearly fewer lanes without work (32-token blocks of 656-byte rows are 5.1 tiles of 256 lanes:
    // 5.1 TB/s; 10.3 tiles of 128 lanes: 5.8).
    if (vec && !plan->threads_chosen && !plan->tuning.variant && threads == kDefaultBlockThreads) {
        auto idle = [&](uint64_t t) { return 1.0 - (double)unit_vecs / (double)((unit_vecs + t - 1) / t * t); };
        if (idle(threads) - idle(threads / 2) > 0.07) threads /= 2;
    }
    // descriptors that fill less than half a workgroup: deal the lanes out without tiles
    if (vec && !plan->tuning.variant && unit_vecs * 2 <= plan->tuning.block_threads) {
        v = pack ? kFlatPackCode : kFlatUnpackCode;
        threads = plan->tuning.block_threads;
    }
    dim3 block(threads);
    if (!vec) {
        // one workgroup per descriptor; a launch holds fewer than 2^32 lanes
        const uint64_t per_launch = kMaxLanesPerLaunch / threads;
        for (uint64_t first = 0; first < a.n_units; first += per_launch) {
            CopyArgs part = a;
            part.unit_begin = a.unit_begin + (uint32_t)first;
            part.n_units = (uint32_t)std::min<uint64_t>(per_launch, a.n_units - first);
            dim3 grid(part.n_units, plane_end - plane_begin);
            if (pack) hipLaunchKernelGGL(kvl_bytes_kernel<true>, grid, block, 0, stream, part);
            else hipLaunchKernelGGL(kvl_bytes_kernel<false>, grid, block, 0, stream, part);
        }
    } else if (v & 128u) {
        // lane indices are 32 bits: split the descriptors over launches where they would not fit
        // (tuning.max_groups, if given, lowers the workgroups per launch further)
        uint64_t lanes_per_launch = (1ull << 32) - threads;
        if (plan->tuning.max_groups)
            lanes_per_launch = std::min<uint64_t>(lanes_per_launch, (uint64_t)plan->tuning.max_groups * threads);
        const uint64_t per_launch = std::max<uint64_t>(1, lanes_per_launch / std::max<uint64_t>(1, unit_vecs));
        for (uint64_t first = 0; first < a.n_units; first += per_launch) {
            CopyArgs part = a;
            part.unit_begin = a.unit_begin + (uint32_t)first;
            part.n_units = (uint32_t)std::min<uint64_t>(per_launch, a.n_units - first);
            const uint64_t lanes = (uint64_t)part.n_units * unit_vecs;
            dim3 grid((uint32_t)((lanes + threads - 1) / threads), plane_end - plane_begin);
            if (pack) launch_flat_variant<true>(v, grid, block, stream, part, plan->max_unit_rows);
            else launch_flat_variant<false>(v, grid, block, stream, part, plan->max_unit_rows);
        }
    } else if ((v & 3u) >= 2u) {
        const uint32_t vpt = (v & 3u) == 3u ? 2 : 1;
        uint32_t max_row = 0;
        for (uint32_t p = plane_begin; p < plane_end; ++p) max_row = std::max(max_row, a.row_elems[p]);
        const uint64_t per_tile = (uint64_t)threads * vpt;
        // destination spans start on 128-byte lines by themselves when the rows and the base do
        bool dst_lines = true;
        for (uint32_t p = plane_begin; p < plane_end; ++p)
            dst_lines = dst_lines && plan->layout.row_bytes[p] % 128 == 0 &&
                        (pack ? a.xfer[p] : a.pool[p]) % 128 == 0;
        const uint32_t al = (dst_lines || (v & 64u)) ? 0u : 1u;
        const uint64_t tpu = ((uint64_t)plan->max_unit_rows * max_row + (al ? 7 : 0) + per_tile - 1) / per_tile;
        const uint64_t blocks = (uint64_t)a.n_units * tpu;
        if (tpu == 0 || blocks > (uint64_t)INT32_MAX) return KVL_ERANGE;
        // fewer workgroups than tiles, each walking over several: on request, or because the
        // far side is host memory
        const uint32_t cap = plan->tuning.max_groups ? plan->tuning.max_groups : (far_host ? kHostSideGroups : 0u);
        if (v & 256u) {
            // pipelined walk: as many workgroups as the machine holds at once (32 wavefronts per compute
            // unit), shared among the planes of the launch
            const uint64_t resident = (uint64_t)compute_units(plan->device) * (2048u / threads);
            uint64_t groups = cap ? cap : std::max<uint64_t>(1, resident / (plane_end - plane_begin));
            groups = std::min<uint64_t>(groups, blocks);
            dim3 grid((uint32_t)groups, plane_end - plane_begin);
            if (pack) launch_pipe_variant<true>(v, grid, block, stream, a, (uint32_t)tpu, al, (uint32_t)blocks);
            else launch_pipe_variant<false>(v, grid, block, stream, a, (uint32_t)tpu, al, (uint32_t)blocks);
            KVL_HIP(hipGetLastError());
            mark_launch(plan, stream);
            return KVL_OK;
        }
        // one workgroup per tile, unless a cap was asked for or the launch would not fit
        bool walk = false;
        const uint32_t groups = launch_groups(blocks, threads, cap, &walk);
        const uint32_t n_tiles = walk ? (uint32_t)blocks : 0u;
        dim3 grid(groups, plane_end - plane_begin);
        if (pack) {
            if (vpt == 2) launch_tile_variant<true, 2>(v, grid, block, stream, a, (uint32_t)tpu, al, n_tiles);
            else launch_tile_variant<true, 1>(v, grid, block, stream, a, (uint32_t)tpu, al, n_tiles);
        } else {
            if (vpt == 2) launch_tile_variant<false, 2>(v, grid, block, stream, a, (uint32_t)tpu, al, n_tiles);
            else launch_tile_variant<false, 1>(v, grid, block, stream, a, (uint32_t)tpu, al, n_tiles);
        }
    } else {
        const uint32_t per_wg = (v & 3u) == 1u ? threads / 64 : 1;
        if ((uint64_t)((a.n_units + per_wg - 1) / per_wg) * threads > kMaxLanesPerLaunch) return KVL_ERANGE;
        dim3 grid((a.n_units + per_wg - 1) / per_wg, plane_end - plane_begin);
        if (pack) launch_span_variant<true>(v, grid, block, stream, a);
        else launch_span_variant<false>(v, grid, block, stream, a);
    }
    KVL_HIP(hipGetLastError());
    mark_launch(plan, stream);
    return KVL_OK;
}

// Launch the layout-converting kernel on descriptors [unit_begin, unit_end).  A
// descriptor of block index k finds its rows at
//   base + k * block_pitch + layer_off + (plane span, row) inside the Layer Block;
// for a buffer of Full Blocks block_pitch is the Full-Block size and layer_off the
// layer's offset in it, for a staging area of Layer Blocks block_pitch is the
// Layer-Block size and layer_off is 0 (base may then lie before the area).
int fullblock_launch(const kvl_plan_t *plan, bool to_pool, uintptr_t base, uint64_t block_pitch,
                     uint64_t layer_off, uint32_t unit_begin, uint32_t unit_end,
                     void *const *pool_planes, hipStream_t stream, bool far_host) {
    if (unit_end <= unit_begin) return KVL_OK;
    if (!plan->d_units || unit_end > plan->units.size()) return KVL_EINVAL;
    const uint32_t P = plan->layout.n_planes;
    const uint64_t bs = plan->layout.block_tokens;
    bool vec = plan->vec16 && base % 16 == 0 && block_pitch % 16 == 0 && layer_off % 16 == 0;
    for (uint32_t p = 0; p < P; ++p) {
        if (!pool_planes[p]) return KVL_EINVAL;
        vec = vec && reinterpret_cast<uintptr_t>(pool_planes[p]) % 16 == 0;
    }
    const uint64_t e = vec ? 16 : 1;          // element size
    FullBlockArgs a{};
    a.units = plan->d_units + unit_begin;
    a.n_units = unit_end - unit_begin;
    a.block_tokens = plan->layout.block_tokens;
    a.blocks = base;
    a.fb_elems = block_pitch / e;
    uint64_t plane_off = 0;
    uint32_t max_row = 0;
    for (uint32_t p = 0; p < P; ++p) {
        a.row_elems[p] = (uint32_t)(plan->layout.row_bytes[p] / e);
        a.pool[p] = reinterpret_cast<uintptr_t>(pool_planes[p]);
        a.layer_plane_off[p] = (layer_off + plane_off) / e;
        plane_off += bs * plan->layout.row_bytes[p];
        max_row = std::max(max_row, a.row_elems[p]);
    }
    const uint32_t threads = 256;
    // across the host link: two elements per lane on few workgroups (as the copy kernels do, see launch_units)
    const uint32_t vpt = far_host ? 2 : 1;
    const uint64_t per_tile = (uint64_t)threads * vpt;
    const uint64_t tpu = ((uint64_t)plan->max_unit_rows * max_row + per_tile - 1) / per_tile;
    const uint64_t wgs = (uint64_t)a.n_units * tpu;
    if (tpu == 0 || wgs > (uint64_t)INT32_MAX) return KVL_ERANGE;
    const uint32_t cap = plan->tuning.max_groups ? plan->tuning.max_groups : (far_host ? kHostSideGroups : 0u);
    const uint32_t n_tiles = (uint32_t)wgs;
    bool walk = false;
    dim3 grid(launch_groups(wgs, threads, cap, &walk), P), block(threads);
#define KVL_FB_LAUNCH(TP, VE, VP) \
    hipLaunchKernelGGL((kvl_fullblock_kernel<TP, VE, VP>), grid, block, 0, stream, a, (uint32_t)tpu, n_tiles)
    if (to_pool) {
        if (vec) { if (vpt == 2) KVL_FB_LAUNCH(true, true, 2); else KVL_FB_LAUNCH(true, true, 1); }
        else { if (vpt == 2) KVL_FB_LAUNCH(true, false, 2); else KVL_FB_LAUNCH(true, false, 1); }
    } else {
        if (vec) { if (vpt == 2) KVL_FB_LAUNCH(false, true, 2); else KVL_FB_LAUNCH(false, true, 1); }
        else { if (vpt == 2) KVL_FB_LAUNCH(false, false, 2); else KVL_FB_LAUNCH(false, false, 1); }
    }
#undef KVL_FB_LAUNCH
    KVL_HIP(hipGetLastError());
    mark_launch(plan, stream);
    return KVL_OK;
}

// Bytes of one Layer Block (all planes of one block, one layer).
uint64_t layer_block_bytes(const kvl_plan_t *plan) {
    uint64_t lb = 0;
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
        lb += (uint64_t)plan->layout.block_tokens * plan->layout.row_bytes[p];
    return lb;
}

// What every Full-Block call asks of its plan and sizes.
int check_fullblock_args(const kvl_plan_t *plan, bool to_pool, uint64_t blocks_bytes, uint32_t layer) {
    if (!plan) return KVL_EINVAL;
    if ((plan->flags & KVL_HOST_ONLY) || !(plan->flags & KVL_NO_MERGE)) return KVL_EINVAL;
    if (!(plan->flags & (to_pool ? KVL_SCATTER : KVL_GATHER))) return KVL_EINVAL;
    if (layer >= plan->layout.n_layers) return KVL_EINVAL;
    const uint64_t fb = layer_block_bytes(plan) * plan->layout.n_layers;
    if (blocks_bytes < plan->blocks_touched * fb) return KVL_ESPACE;
    return KVL_OK;
}

int fullblock_layer(const kvl_plan_t *plan, bool to_pool, uintptr_t blocks, uint64_t blocks_bytes,
                    uint32_t layer, void *const *pool_planes, hipStream_t stream) {
    if (!pool_planes) return KVL_EINVAL;
    int rc = check_fullblock_args(plan, to_pool, blocks_bytes, layer);
    if (rc != KVL_OK) return rc;
    if (plan->units.empty()) return KVL_OK;
    if (!blocks) return KVL_EINVAL;
    const uint64_t lb = layer_block_bytes(plan), fb = lb * plan->layout.n_layers;
    rc = check_device(plan);
    if (rc == KVL_OK) rc = check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK)
        rc = check_buffer(plan, reinterpret_cast<const void *>(blocks), plan->blocks_touched * fb, true);
    if (rc != KVL_OK) return rc;
    return fullblock_launch(plan, to_pool, blocks, fb, (uint64_t)layer * lb, 0, (uint32_t)plan->units.size(),
                            pool_planes, stream, is_host_memory(plan, reinterpret_cast<const void *>(blocks)));
}

}  // namespace kvl

extern "C" {

int kvl_fullblocks_to_pool_layer(const kvl_plan_t *plan, const void *full_blocks, uint64_t full_blocks_bytes,
                                 uint32_t layer, void *const *pool_planes, void *stream) {
    return kvl::fullblock_layer(plan, true, reinterpret_cast<uintptr_t>(full_blocks), full_blocks_bytes, layer,
                                pool_planes, (hipStream_t)stream);
}

int kvl_pool_to_fullblocks_layer(const kvl_plan_t *plan, const void *const *pool_planes, uint32_t layer,
                                 void *full_blocks, uint64_t full_blocks_bytes, void *stream) {
    return kvl::fullblock_layer(plan, false, reinterpret_cast<uintptr_t>(full_blocks), full_blocks_bytes, layer,
                                const_cast<void *const *>(pool_planes), (hipStream_t)stream);
}

int kvl_move_layer(const kvl_plan_t *plan, const void *const *src_pool_planes, void *const *dst_pool_planes,
                   void *stream) {
    if (!plan || !src_pool_planes || !dst_pool_planes) return KVL_EINVAL;
    if (!plan->paired || (plan->flags & KVL_HOST_ONLY)) return KVL_EINVAL;
    if (plan->units.empty()) return KVL_OK;
    int rc = kvl::check_pool(plan, src_pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = kvl::check_pool(plan, dst_pool_planes, plan->dst_pool_blocks);
    if (rc != KVL_OK) return rc;
    // the gather kernel with the destination pool in the transfer buffer's place:
    // a paired descriptor's xfer_row is a row of the destination pool
    uintptr_t xp[KVL_MAX_PLANES];
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p) {
        if (!dst_pool_planes[p]) return KVL_EINVAL;
        xp[p] = reinterpret_cast<uintptr_t>(dst_pool_planes[p]);
    }
    return kvl::launch_units(plan, true, 0, (uint32_t)plan->units.size(), 0, plan->layout.n_planes,
                             const_cast<void *const *>(src_pool_planes), xp, (hipStream_t)stream);
}

int kvl_pack_layer(const kvl_plan_t *plan, const void *const *pool_planes, void *xfer,
                   uint64_t xfer_capacity, void *stream) {
    if (!plan || !pool_planes) return KVL_EINVAL;
    if (!(plan->flags & KVL_GATHER) || (plan->flags & KVL_HOST_ONLY) || plan->paired) return KVL_EINVAL;
    if (xfer_capacity < plan->payload_bytes) return KVL_ESPACE;
    if (plan->units.empty()) return KVL_OK;
    if (!xfer) return KVL_EINVAL;
    int rc = kvl::check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = kvl::check_buffer(plan, xfer, plan->payload_bytes, true);
    if (rc != KVL_OK) return rc;
    uintptr_t xp[KVL_MAX_PLANES];
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
        xp[p] = reinterpret_cast<uintptr_t>(xfer) + plan->plane_base[p];
    return kvl::launch_units(plan, true, 0, (uint32_t)plan->units.size(), 0, plan->layout.n_planes,
                             const_cast<void *const *>(pool_planes), xp, (hipStream_t)stream,
                             kvl::is_host_memory(plan, xfer));
}

int kvl_unpack_layer(const kvl_plan_t *plan, const void *xfer, uint64_t xfer_bytes,
                     void *const *pool_planes, void *stream) {
    if (!plan || !pool_planes) return KVL_EINVAL;
    if (!(plan->flags & KVL_SCATTER) || (plan->flags & KVL_HOST_ONLY)) return KVL_EINVAL;
    if (xfer_bytes < plan->payload_bytes) return KVL_ESPACE;
    if (plan->units.empty()) return KVL_OK;
    if (!xfer) return KVL_EINVAL;
    int rc = kvl::check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = kvl::check_buffer(plan, xfer, plan->payload_bytes, true);
    if (rc != KVL_OK) return rc;
    uintptr_t xp[KVL_MAX_PLANES];
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
        xp[p] = reinterpret_cast<uintptr_t>(xfer) + plan->plane_base[p];
    return kvl::launch_units(plan, false, 0, (uint32_t)plan->units.size(), 0, plan->layout.n_planes,
                             pool_planes, xp, (hipStream_t)stream, kvl::is_host_memory(plan, xfer));
}

int kvl_copy_linear(const void *src, void *dst, uint64_t bytes, void *stream) {
    if (bytes == 0) return KVL_OK;
    if (!src || !dst) return KVL_EINVAL;
    if (bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16)
        return KVL_EINVAL;
    int rc = kvl_check_buffer(src, bytes, 1);
    if (rc == KVL_OK) rc = kvl_check_buffer(dst, bytes, 1);
    if (rc != KVL_OK) return rc;
    // a launch holds fewer than 2^32 lanes: larger copies go in several
    const uint64_t n = bytes / 16, per_launch = (kvl::kMaxLanesPerLaunch / 256) * 256;
    for (uint64_t first = 0; first < n; first += per_launch) {
        const uint64_t m = std::min<uint64_t>(per_launch, n - first);
        hipLaunchKernelGGL(kvl::kvl_linear_kernel, dim3((uint32_t)((m + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                           static_cast<const kvl::v4u *>(src) + first, static_cast<kvl::v4u *>(dst) + first, m);
        KVL_HIP(hipGetLastError());
    }
    return KVL_OK;
}

int kvl_ceiling_kernel(const kvl_ceiling_t *c, const void *src, uint64_t src_bytes, void *dst, uint64_t dst_bytes,
                       uint64_t bytes, const uint32_t *block_table, void *stream) {
    using namespace kvl;
    if (!c || !src || !dst || bytes == 0) return KVL_EINVAL;
    if (c->mode > KVL_CEILING_WRITE || c->skew_bytes % 16 || c->skew_bytes >= 128 || c->block_bytes % 16) return KVL_EINVAL;
    if (bytes % 16 || reinterpret_cast<uintptr_t>(src) % 128 || reinterpret_cast<uintptr_t>(dst) % 128) return KVL_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    if (c->block_bytes == 0) {
        // one linear stream; the skew shifts the source
        if (src_bytes < bytes + c->skew_bytes || dst_bytes < bytes) return KVL_ESPACE;
        int rc = kvl_check_buffer(src, bytes + c->skew_bytes, 0);
        if (rc == KVL_OK) rc = kvl_check_buffer(dst, bytes, 0);
        if (rc != KVL_OK) return rc;
        const uint64_t n = bytes / 16, per_launch = (kMaxLanesPerLaunch / 256) * 256;
        const v4u *from = reinterpret_cast<const v4u *>(static_cast<const char *>(src) + c->skew_bytes);
        for (uint64_t first = 0; first < n; first += per_launch) {
            const uint64_t m = std::min<uint64_t>(per_launch, n - first);
            const dim3 grid((uint32_t)((m + 255) / 256)), block(256);
            v4u *to = static_cast<v4u *>(dst) + first;
            if (c->mode == KVL_CEILING_COPY)
                hipLaunchKernelGGL((kvl_ceiling_linear_kernel<0, kLinearNtLoad, kLinearStorePolicy>), grid, block, 0, s, from + first, to, m);
            else if (c->mode == KVL_CEILING_READ)
                hipLaunchKernelGGL((kvl_ceiling_linear_kernel<1, kLinearNtLoad, kLinearStorePolicy>), grid, block, 0, s, from + first, to, m);
            else
                hipLaunchKernelGGL((kvl_ceiling_linear_kernel<2, kLinearNtLoad, kLinearStorePolicy>), grid, block, 0, s, from + first, to, m);
            KVL_HIP(hipGetLastError());
        }
        return KVL_OK;
    }
    if (bytes % c->block_bytes || c->hop_blocks_log2 > 31) return KVL_EINVAL;
    const uint64_t n_blocks = bytes / c->block_bytes, hop_blocks = 1ull << c->hop_blocks_log2;
    if (n_blocks > hop_blocks || n_blocks > UINT32_MAX) return KVL_EINVAL;
    const uint64_t hop_bytes = hop_blocks * c->block_bytes, dense_bytes = bytes + c->skew_bytes;
    const bool gather = c->hopping_side == 0;
    if ((gather ? src_bytes : dst_bytes) < hop_bytes || (gather ? dst_bytes : src_bytes) < dense_bytes) return KVL_ESPACE;
    int rc = kvl_check_buffer(src, gather ? hop_bytes : dense_bytes, 0);
    if (rc == KVL_OK) rc = kvl_check_buffer(dst, gather ? dense_bytes : hop_bytes, 0);
    if (rc == KVL_OK && block_table) rc = kvl_check_buffer(block_table, n_blocks * 4, 0);
    if (rc != KVL_OK) return rc;
    CeilingArgs a{};
    a.dense = reinterpret_cast<uintptr_t>(gather ? dst : src);
    a.hopping = reinterpret_cast<uintptr_t>(gather ? const_cast<void *>(src) : dst);
    a.table = block_table;
    a.n_blocks = (uint32_t)n_blocks;
    a.hop_mask = (uint32_t)(hop_blocks - 1);
    a.mul = 0x9e3779b1u;                    // odd
    a.block_vecs = c->block_bytes / 16;
    a.tiles_per_block = (a.block_vecs + 7 + 255) / 256;
    a.skew_vecs = c->skew_bytes / 16;
    a.tile_magic = ((1ull << 40) + a.tiles_per_block - 1) / a.tiles_per_block;
    const uint64_t groups = n_blocks * a.tiles_per_block;
    // the multiplication finds the block of every workgroup index below 2^24 * tiles_per_block exactly
    if (groups > (1ull << 24) || groups * 256 > kMaxLanesPerLaunch) return KVL_ERANGE;
    const dim3 grid((uint32_t)groups), block(256);
#define KVL_CEIL(M, G, N, S) hipLaunchKernelGGL((kvl_ceiling_pattern_kernel<M, G, N, S>), grid, block, 0, s, a)
    // the cache policies of the default gather and scatter
    if (gather) {
        if (c->mode == KVL_CEILING_COPY) KVL_CEIL(0, true, true, 2);
        else if (c->mode == KVL_CEILING_READ) KVL_CEIL(1, true, true, 2);
        else KVL_CEIL(2, true, true, 2);
    } else {
        if (c->mode == KVL_CEILING_COPY) KVL_CEIL(0, false, false, 3);
        else if (c->mode == KVL_CEILING_READ) KVL_CEIL(1, false, false, 3);
        else KVL_CEIL(2, false, false, 3);
    }
#undef KVL_CEIL
    KVL_HIP(hipGetLastError());
    return KVL_OK;
}

const char *kvl_variant_name(uint32_t v) {
    static thread_local char name[64];
    if (v == 0) return "default";
    if (v > kvl::kNumVariants) return nullptr;
    v -= 1;
    static const char *modes[4] = {"wg/unit", "wave/unit", "tile x1", "tile x2"};
    static const char *sp[4] = {"", " st:nt", " st:sc1", " st:sc1+nt"};
    if (v & 256u)
        std::snprintf(name, sizeof name, "pipe%s%s%s", (v & 4u) ? " ld:nt" : "", sp[(v >> 3) & 3u],
                      (v & 64u) ? " noalign" : "");
    else if (v & 128u)
        std::snprintf(name, sizeof name, "flat%s%s", (v & 4u) ? " ld:nt" : "", sp[(v >> 3) & 3u]);
    else
        std::snprintf(name, sizeof name, "%s%s%s%s%s", modes[v & 3u], (v & 4u) ? " ld:nt" : "",
                      sp[(v >> 3) & 3u], (v & 32u) ? " deep" : "", (v & 64u) ? " noalign" : "");
    return name;
}

}  // extern "C"
