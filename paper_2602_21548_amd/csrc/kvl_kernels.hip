// Device side of pack / unpack: copy kernels for gfx950 and their launchers.
//
// The work is pure data movement (no arithmetic on the payload).  A copy
// descriptor names a span of token rows that is contiguous in the paged pool and
// in the transfer buffer, so each descriptor is a straight 16-byte-vector copy;
// what the block table fragments is only where each span starts.  The kernels
// therefore read a descriptor (wave-uniform, through the scalar cache), form two
// 64-bit addresses and stream the span with several 16-byte loads in flight per
// lane before the matching stores.  Consecutive lanes touch consecutive 16-byte
// vectors, so every wavefront load or store covers 1 KiB of contiguous memory.
//
// kvl_tuning_t::variant is 0 for the default below, else 1 + code with
// code = mode | ntl << 2 | sp << 3 | deep << 5 | noalign << 6:
//   mode 0  one workgroup per descriptor, each lane loops over the span
//   mode 1  one wavefront per descriptor, each lane loops over the span
//   mode 2  tiled: a descriptor is cut into tiles of blockDim vectors and every
//           lane moves exactly one 16-byte vector
//   mode 3  tiled, two vectors per lane
//   ntl     non-temporal loads
//   sp      store cache policy: 0 plain, 1 nt, 2 sc1, 3 sc1 nt
//   deep    modes 0-1: 8 instead of 4 vectors in flight per lane
//   noalign modes 2-3: do not line tiles up with the destination's 128-byte lines
//           (they are lined up by default whenever the rows are not multiples of 128 bytes)
// Measured on MI355X (5.2 GB of 72 KiB blocks in random order), the tiled form
// with one vector per lane and 256-lane workgroups is the fastest: it leaves no
// dependency between a lane's memory operations and lets the hardware fill the
// memory system with resident wavefronts.  Cache policies, measured with gather
// and scatter alternating as they do in use: the gather (random reads,
// sequential writes) runs best with non-temporal loads and sc1 stores; the
// scatter (sequential reads, random writes) with sc1+nt stores, and with
// non-temporal loads only if the rows are multiples of 128 bytes (otherwise
// neighbouring wavefronts share source lines, and a non-temporal load fetches
// the shared line twice).  Together the policies are worth 5-15 % over plain
// loads and stores.  With rows that are not multiples of 128 bytes the tiles are
// also lined up with the destination's cache lines (worth 5-9 % on 656-byte rows).
#include <algorithm>
#include <cstdio>

#include "kvl_internal.h"

namespace kvl {

// default variant codes (see the list above) and the plain copy's policies
constexpr uint32_t kDefaultPackCode = 2u | 4u | (2u << 3);   // tile x1, nt loads, sc1 stores
constexpr uint32_t kDefaultUnpackCode = 2u | 4u | (3u << 3);    // tile x1, nt loads, sc1+nt stores
constexpr uint32_t kDefaultUnpackCodeOddRows = 2u | (3u << 3);  // tile x1, plain loads, sc1+nt stores
constexpr bool kLinearNtLoad = true;
constexpr int kLinearStorePolicy = 2;

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
// Every buffer is device (or device-mapped) memory: say so, so that the
// compiler emits global_load / global_store rather than flat accesses.
typedef const v4u __attribute__((address_space(1))) *gsrc_t;
typedef v4u __attribute__((address_space(1))) *gdst_t;

struct CopyArgs {
    const kvl_unit_t *units;       // device descriptors
    uint32_t unit_begin;           // first descriptor of this launch
    uint32_t n_units;              // descriptors in this launch
    uint32_t plane_begin;          // blockIdx.y + plane_begin is the plane
    uint32_t row_elems[KVL_MAX_PLANES];  // row size in 16-byte vectors (vector kernels) or bytes
    uintptr_t pool[KVL_MAX_PLANES];      // plane base of the paged pool
    uintptr_t xfer[KVL_MAX_PLANES];      // address of transfer row 0 of the plane
};

// The descriptors live on the device that was current when the plan was made.
static int check_device(const kvl_plan_t *plan) {
    int dev = -1;
    KVL_HIP(hipGetDevice(&dev));
    return dev == plan->device ? KVL_OK : KVL_EINVAL;
}

template <bool NT>
__device__ __forceinline__ v4u load16(gsrc_t p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

// Store with a cache policy.  The compiler only offers the non-temporal hint;
// the system-scope write-through forms (sc1) are written out as instructions.
// A store needs no wait: nothing here reads what it wrote.
template <int SP>
__device__ __forceinline__ void store16(gdst_t p, v4u v) {
    if (SP == 0) *p = v;
    else if (SP == 1) __builtin_nontemporal_store(v, p);
    else if (SP == 2) asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
    else asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
}

// `lanes` threads copy n 16-byte vectors; this thread is `lane`.  U loads are
// issued before the first store so that U KiB per wavefront are in flight.
template <int U, bool NTL, int SP>
__device__ __forceinline__ void copy_span(gsrc_t __restrict__ src, gdst_t __restrict__ dst,
                                          uint32_t n, uint32_t lane, uint32_t lanes) {
    // n is below 2^32: a descriptor never spans more than 1 GiB
    const uint32_t step = lanes * U;
    const uint32_t last = lanes * (U - 1);
    uint32_t i = lane;
    // no division: a lane takes a full step while its last vector is in range
    for (; (uint64_t)i + last < n; i += step) {
        v4u v[U];
#pragma unroll
        for (int k = 0; k < U; ++k) v[k] = load16<NTL>(src + i + k * lanes);
#pragma unroll
        for (int k = 0; k < U; ++k) store16<SP>(dst + i + k * lanes, v[k]);
    }
    // ragged tail: this lane has at most U-1 vectors left
    v4u v[U];
#pragma unroll
    for (int k = 0; k < U - 1; ++k) {
        const uint64_t j = (uint64_t)i + (uint64_t)k * lanes;
        if (j < n) v[k] = load16<NTL>(src + j);
    }
#pragma unroll
    for (int k = 0; k < U - 1; ++k) {
        const uint64_t j = (uint64_t)i + (uint64_t)k * lanes;
        if (j < n) store16<SP>(dst + j, v[k]);
    }
}

template <bool PACK, bool WAVE, int U, bool NTL, int SP>
__device__ __forceinline__ void units_body(const CopyArgs &a) {
    uint32_t u_idx, lane, lanes;
    if (WAVE) {
        const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        u_idx = blockIdx.x * (blockDim.x >> 6) + wave;
        lane = threadIdx.x & 63u;
        lanes = 64;
    } else {
        u_idx = blockIdx.x;
        lane = threadIdx.x;
        lanes = blockDim.x;
    }
    if (u_idx >= a.n_units) return;
    const kvl_unit_t u = a.units[a.unit_begin + u_idx];
    const uint32_t p = a.plane_begin + blockIdx.y;
    const uint64_t row = a.row_elems[p];
    const uintptr_t pool = a.pool[p] + (uint64_t)u.pool_row * row * 16u;
    const uintptr_t xfer = a.xfer[p] + (uint64_t)u.xfer_row * row * 16u;
    const uint32_t n = u.n_rows * (uint32_t)row;
    if (PACK) copy_span<U, NTL, SP>((gsrc_t)pool, (gdst_t)xfer, n, lane, lanes);
    else copy_span<U, NTL, SP>((gsrc_t)xfer, (gdst_t)pool, n, lane, lanes);
}

// gather: paged pool -> transfer buffer
template <bool WAVE, int U, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_pack_kernel(const CopyArgs a) {
    units_body<true, WAVE, U, NTL, SP>(a);
}

// scatter: transfer buffer -> paged pool
template <bool WAVE, int U, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_unpack_kernel(const CopyArgs a) {
    units_body<false, WAVE, U, NTL, SP>(a);
}

// Tiled form: the grid is (descriptors x tiles_per_unit, planes); a workgroup
// takes tile `t` of its descriptor and each lane moves VPT vectors.  With one
// vector per lane there is no loop and no dependency between a lane's memory
// operations: the hardware keeps the memory system busy by the sheer number of
// resident wavefronts rather than by unrolling.
template <bool PACK, int VPT, bool NTL, int SP>
__device__ __forceinline__ void tile_body(const CopyArgs &a, uint32_t tiles_per_unit, uint32_t align_dst) {
    const uint32_t u_idx = blockIdx.x / tiles_per_unit;
    const uint32_t tile = blockIdx.x - u_idx * tiles_per_unit;
    const kvl_unit_t u = a.units[a.unit_begin + u_idx];
    const uint32_t p = a.plane_begin + blockIdx.y;
    const uint32_t row = a.row_elems[p];
    const uint32_t n = u.n_rows * row;
    const uintptr_t pool = a.pool[p] + (uint64_t)u.pool_row * row * 16u;
    const uintptr_t xfer = a.xfer[p] + (uint64_t)u.xfer_row * row * 16u;
    gsrc_t src = (gsrc_t)(PACK ? pool : xfer);
    gdst_t dst = (gdst_t)(PACK ? xfer : pool);
    // With rows that are not multiples of 128 bytes a span starts anywhere in a
    // cache line.  Tiles are then laid from the 128-byte boundary below the
    // span's first destination byte, so that every wavefront's store covers
    // whole lines (its load may straddle them, which costs far less): the first
    // `lead` lanes of the first tile idle.
    const uint32_t lead = align_dst ? ((uint32_t)((PACK ? xfer : pool) >> 4) & 7u) : 0u;
    const uint32_t first = tile * (blockDim.x * VPT);
    if (first >= n + lead) return;
    v4u v[VPT];
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const uint32_t pos = first + k * blockDim.x + threadIdx.x;
        if (pos >= lead && pos - lead < n) v[k] = load16<NTL>(src + (pos - lead));
    }
#pragma unroll
    for (int k = 0; k < VPT; ++k) {
        const uint32_t pos = first + k * blockDim.x + threadIdx.x;
        if (pos >= lead && pos - lead < n) store16<SP>(dst + (pos - lead), v[k]);
    }
}

template <int VPT, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_pack_tile_kernel(const CopyArgs a, uint32_t tiles_per_unit,
                                                             uint32_t align_dst) {
    tile_body<true, VPT, NTL, SP>(a, tiles_per_unit, align_dst);
}

template <int VPT, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_unpack_tile_kernel(const CopyArgs a, uint32_t tiles_per_unit,
                                                               uint32_t align_dst) {
    tile_body<false, VPT, NTL, SP>(a, tiles_per_unit, align_dst);
}

// Fallback for row sizes or addresses that are not multiples of 16 bytes: one
// workgroup per descriptor, byte by byte.  Correct for any layout, not fast.
template <bool PACK>
__global__ void __launch_bounds__(1024) kvl_bytes_kernel(const CopyArgs a) {
    const kvl_unit_t u = a.units[a.unit_begin + blockIdx.x];
    const uint32_t p = a.plane_begin + blockIdx.y;
    const uint64_t row = a.row_elems[p];
    uint8_t *pool = reinterpret_cast<uint8_t *>(a.pool[p]) + (uint64_t)u.pool_row * row;
    uint8_t *xfer = reinterpret_cast<uint8_t *>(a.xfer[p]) + (uint64_t)u.xfer_row * row;
    const uint64_t n = (uint64_t)u.n_rows * row;
    for (uint64_t i = threadIdx.x; i < n; i += blockDim.x) {
        if (PACK) xfer[i] = pool[i];
        else pool[i] = xfer[i];
    }
}

// Storage layout <-> paged pool for one layer.  Same tiling as above; the far
// side is a buffer of Full Blocks ([layer, tokens, bytes] per block), so a
// descriptor (which never spans blocks here) lands at
//   block_index * FB + (layer, plane) offset + row-in-block * row.
// The buffer may be pinned host memory: then these accesses cross the host link.
struct FullBlockArgs {
    const kvl_unit_t *units;
    uint32_t n_units;
    uint32_t block_tokens;
    uint32_t row_elems[KVL_MAX_PLANES];       // 16-byte vectors (VEC) or bytes per row
    uintptr_t pool[KVL_MAX_PLANES];
    uintptr_t blocks;                          // base of the Full-Block buffer
    uint64_t fb_elems;                         // elements per Full Block
    uint64_t layer_plane_off[KVL_MAX_PLANES];  // element offset of (layer, plane) inside a Full Block
};

template <bool TO_POOL, bool VEC>
__global__ void __launch_bounds__(256) kvl_fullblock_kernel(const FullBlockArgs a, uint32_t tiles_per_unit) {
    const uint32_t u_idx = blockIdx.x / tiles_per_unit;
    const uint32_t tile = blockIdx.x - u_idx * tiles_per_unit;
    const kvl_unit_t u = a.units[u_idx];
    const uint32_t p = blockIdx.y;
    const uint32_t row = a.row_elems[p];
    const uint32_t n = u.n_rows * row;
    const uint32_t i = tile * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t within = u.pool_row % a.block_tokens;
    const uint64_t in_pool = (uint64_t)u.pool_row * row + i;
    const uint64_t in_blocks = (uint64_t)u.block_index * a.fb_elems + a.layer_plane_off[p] +
                               (uint64_t)within * row + i;
    if (VEC) {
        if (TO_POOL) store16<3>((gdst_t)a.pool[p] + in_pool, load16<false>((gsrc_t)a.blocks + in_blocks));
        else store16<0>((gdst_t)a.blocks + in_blocks, load16<true>((gsrc_t)a.pool[p] + in_pool));
    } else {
        uint8_t *pool = reinterpret_cast<uint8_t *>(a.pool[p]);
        uint8_t *blocks = reinterpret_cast<uint8_t *>(a.blocks);
        if (TO_POOL) pool[in_pool] = blocks[in_blocks];
        else blocks[in_blocks] = pool[in_pool];
    }
}

// Straight copy, one vector per lane: the tiled kernel without descriptors.
__global__ void __launch_bounds__(256) kvl_linear_kernel(const v4u *src, v4u *dst, uint64_t n) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) store16<kLinearStorePolicy>((gdst_t)dst + i, load16<kLinearNtLoad>((gsrc_t)src + i));
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

template <bool PACK, int VPT, bool NTL, int SP>
static void launch_tile_one(dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu, uint32_t al) {
    if (PACK) hipLaunchKernelGGL((kvl_pack_tile_kernel<VPT, NTL, SP>), g, b, 0, s, a, tpu, al);
    else hipLaunchKernelGGL((kvl_unpack_tile_kernel<VPT, NTL, SP>), g, b, 0, s, a, tpu, al);
}

template <bool PACK, int VPT, bool NTL>
static void launch_tile_sp(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu,
                           uint32_t al) {
    switch ((v >> 3) & 3u) {
        case 0: launch_tile_one<PACK, VPT, NTL, 0>(g, b, s, a, tpu, al); break;
        case 1: launch_tile_one<PACK, VPT, NTL, 1>(g, b, s, a, tpu, al); break;
        case 2: launch_tile_one<PACK, VPT, NTL, 2>(g, b, s, a, tpu, al); break;
        default: launch_tile_one<PACK, VPT, NTL, 3>(g, b, s, a, tpu, al); break;
    }
}

template <bool PACK, int VPT>
static void launch_tile_variant(uint32_t v, dim3 g, dim3 b, hipStream_t s, const CopyArgs &a, uint32_t tpu,
                                uint32_t al) {
    if (v & 4u) launch_tile_sp<PACK, VPT, true>(v, g, b, s, a, tpu, al);
    else launch_tile_sp<PACK, VPT, false>(v, g, b, s, a, tpu, al);
}

int launch_units(const kvl_plan_t *plan, bool pack, uint32_t unit_begin, uint32_t unit_end,
                 uint32_t plane_begin, uint32_t plane_end,
                 void *const *pool_planes, const uintptr_t *xfer_plane, hipStream_t stream) {
    if (unit_end <= unit_begin || plane_end <= plane_begin) return KVL_OK;
    if (!plan->d_units || unit_end > plan->units.size() || plane_end > plan->layout.n_planes)
        return KVL_EINVAL;
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

    const uint32_t threads = plan->tuning.block_threads;
    // default: tiled, one vector per lane; cache policies as measured (see the top of this file)
    uint32_t v;
    if (plan->tuning.variant) {
        v = plan->tuning.variant - 1;
    } else {
        bool rows_128 = true;       // every span starts on a 128-byte line of the transfer buffer
        for (uint32_t p = plane_begin; p < plane_end; ++p)
            rows_128 = rows_128 && plan->layout.row_bytes[p] % 128 == 0;
        if (pack) v = kDefaultPackCode;
        else v = rows_128 ? kDefaultUnpackCode : kDefaultUnpackCodeOddRows;
    }
    dim3 block(threads);
    if (!vec) {
        dim3 grid(a.n_units, plane_end - plane_begin);
        if (pack) hipLaunchKernelGGL(kvl_bytes_kernel<true>, grid, block, 0, stream, a);
        else hipLaunchKernelGGL(kvl_bytes_kernel<false>, grid, block, 0, stream, a);
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
        dim3 grid((uint32_t)blocks, plane_end - plane_begin);
        if (pack) {
            if (vpt == 2) launch_tile_variant<true, 2>(v, grid, block, stream, a, (uint32_t)tpu, al);
            else launch_tile_variant<true, 1>(v, grid, block, stream, a, (uint32_t)tpu, al);
        } else {
            if (vpt == 2) launch_tile_variant<false, 2>(v, grid, block, stream, a, (uint32_t)tpu, al);
            else launch_tile_variant<false, 1>(v, grid, block, stream, a, (uint32_t)tpu, al);
        }
    } else {
        const uint32_t per_wg = (v & 3u) == 1u ? threads / 64 : 1;
        dim3 grid((a.n_units + per_wg - 1) / per_wg, plane_end - plane_begin);
        if (pack) launch_span_variant<true>(v, grid, block, stream, a);
        else launch_span_variant<false>(v, grid, block, stream, a);
    }
    KVL_HIP(hipGetLastError());
    return KVL_OK;
}

int fullblock_layer(const kvl_plan_t *plan, bool to_pool, uintptr_t blocks, uint64_t blocks_bytes,
                           uint32_t layer, void *const *pool_planes, hipStream_t stream) {
    if (!plan || !pool_planes) return KVL_EINVAL;
    if ((plan->flags & KVL_HOST_ONLY) || !(plan->flags & KVL_NO_MERGE)) return KVL_EINVAL;
    if (!(plan->flags & (to_pool ? KVL_SCATTER : KVL_GATHER))) return KVL_EINVAL;
    if (layer >= plan->layout.n_layers) return KVL_EINVAL;
    const uint32_t P = plan->layout.n_planes;
    const uint64_t bs = plan->layout.block_tokens;
    uint64_t lb = 0;
    for (uint32_t p = 0; p < P; ++p) lb += bs * plan->layout.row_bytes[p];
    const uint64_t fb = lb * plan->layout.n_layers;
    if (blocks_bytes < plan->blocks_touched * fb) return KVL_ESPACE;
    if (plan->units.empty()) return KVL_OK;
    if (!blocks) return KVL_EINVAL;
    int rc_dev = check_device(plan);
    if (rc_dev != KVL_OK) return rc_dev;
    bool vec = plan->vec16 && blocks % 16 == 0;
    for (uint32_t p = 0; p < P; ++p) {
        if (!pool_planes[p]) return KVL_EINVAL;
        vec = vec && reinterpret_cast<uintptr_t>(pool_planes[p]) % 16 == 0;
    }
    const uint64_t e = vec ? 16 : 1;          // element size
    FullBlockArgs a{};
    a.units = plan->d_units;
    a.n_units = (uint32_t)plan->units.size();
    a.block_tokens = plan->layout.block_tokens;
    a.blocks = blocks;
    a.fb_elems = fb / e;
    uint64_t plane_off = 0;
    uint32_t max_row = 0;
    for (uint32_t p = 0; p < P; ++p) {
        a.row_elems[p] = (uint32_t)(plan->layout.row_bytes[p] / e);
        a.pool[p] = reinterpret_cast<uintptr_t>(pool_planes[p]);
        a.layer_plane_off[p] = ((uint64_t)layer * lb + plane_off) / e;
        plane_off += bs * plan->layout.row_bytes[p];
        max_row = std::max(max_row, a.row_elems[p]);
    }
    const uint32_t threads = 256;
    const uint64_t tpu = ((uint64_t)plan->max_unit_rows * max_row + threads - 1) / threads;
    const uint64_t wgs = (uint64_t)a.n_units * tpu;
    if (tpu == 0 || wgs > (uint64_t)INT32_MAX) return KVL_ERANGE;
    dim3 grid((uint32_t)wgs, P), block(threads);
    if (to_pool) {
        if (vec) hipLaunchKernelGGL((kvl_fullblock_kernel<true, true>), grid, block, 0, stream, a, (uint32_t)tpu);
        else hipLaunchKernelGGL((kvl_fullblock_kernel<true, false>), grid, block, 0, stream, a, (uint32_t)tpu);
    } else {
        if (vec) hipLaunchKernelGGL((kvl_fullblock_kernel<false, true>), grid, block, 0, stream, a, (uint32_t)tpu);
        else hipLaunchKernelGGL((kvl_fullblock_kernel<false, false>), grid, block, 0, stream, a, (uint32_t)tpu);
    }
    KVL_HIP(hipGetLastError());
    return KVL_OK;
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
    uintptr_t xp[KVL_MAX_PLANES];
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
        xp[p] = reinterpret_cast<uintptr_t>(xfer) + plan->plane_base[p];
    return kvl::launch_units(plan, true, 0, (uint32_t)plan->units.size(), 0, plan->layout.n_planes,
                             const_cast<void *const *>(pool_planes), xp, (hipStream_t)stream);
}

int kvl_unpack_layer(const kvl_plan_t *plan, const void *xfer, uint64_t xfer_bytes,
                     void *const *pool_planes, void *stream) {
    if (!plan || !pool_planes) return KVL_EINVAL;
    if (!(plan->flags & KVL_SCATTER) || (plan->flags & KVL_HOST_ONLY)) return KVL_EINVAL;
    if (xfer_bytes < plan->payload_bytes) return KVL_ESPACE;
    if (plan->units.empty()) return KVL_OK;
    if (!xfer) return KVL_EINVAL;
    uintptr_t xp[KVL_MAX_PLANES];
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
        xp[p] = reinterpret_cast<uintptr_t>(xfer) + plan->plane_base[p];
    return kvl::launch_units(plan, false, 0, (uint32_t)plan->units.size(), 0, plan->layout.n_planes,
                             pool_planes, xp, (hipStream_t)stream);
}

int kvl_copy_linear(const void *src, void *dst, uint64_t bytes, void *stream) {
    if (bytes == 0) return KVL_OK;
    if (!src || !dst) return KVL_EINVAL;
    if (bytes % 16 || reinterpret_cast<uintptr_t>(src) % 16 || reinterpret_cast<uintptr_t>(dst) % 16)
        return KVL_EINVAL;
    const uint64_t n = bytes / 16;
    const uint64_t blocks = (n + 255) / 256;
    if (blocks > (uint64_t)INT32_MAX) return KVL_ERANGE;
    hipLaunchKernelGGL(kvl::kvl_linear_kernel, dim3((uint32_t)blocks), dim3(256), 0, (hipStream_t)stream,
                       static_cast<const kvl::v4u *>(src), static_cast<kvl::v4u *>(dst), n);
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
    std::snprintf(name, sizeof name, "%s%s%s%s%s", modes[v & 3u], (v & 4u) ? " ld:nt" : "",
                  sp[(v >> 3) & 3u], (v & 32u) ? " deep" : "", (v & 64u) ? " noalign" : "");
    return name;
}

}  // extern "C"
