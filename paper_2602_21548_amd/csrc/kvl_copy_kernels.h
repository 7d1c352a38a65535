// Device code of the copy kernels (gfx950).  Included by kvl_kernels.hip only.
//
// The work is pure data movement (no arithmetic on the payload).  A copy
// descriptor names a span of token rows that is contiguous in the paged pool and
// in the transfer buffer, so each descriptor is a straight 16-byte-vector copy;
// what the block table fragments is only where each span starts.  The kernels
// therefore read a descriptor (wave-uniform, through the scalar cache), form two
// 64-bit addresses and either move one 16-byte vector per lane (the tiled form,
// the default) or loop over the span with several loads in flight per lane.
// Consecutive lanes touch consecutive 16-byte vectors, so every wavefront load
// or store covers 1 KiB of contiguous memory.
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
//   pipe    (code bit 8, with ntl, sp and noalign only) the tiled form on a fixed grid of resident
//           workgroups, each walking over its tiles with loads, stores and descriptor fetches
//           software-pipelined (see kvl_tile_pipe_kernel)
//   flat    (code bit 7, with ntl and sp only) no tiles: lane g of the launch takes vector
//           g mod m of descriptor g div m, m = vectors of the largest descriptor; for
//           descriptors far smaller than a workgroup (token-granular pools)
// The default is the tiled form, or the flat one when the largest descriptor fills less
// than half a workgroup: on 2 M single-token blocks of 1152 bytes the tiled form leaves
// 72 % of its lanes idle and the flat one keeps all of them busy (gather 3.2 -> 5.3 TB/s;
// the scatter stays at 3.3-3.7 TB/s in every form: random 1152-byte writes are the
// memory's limit there, 1 KiB ones reach 4.5-4.7).
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
#pragma once

#include "kvl_internal.h"

namespace kvl {

// default variant codes (see the list above) and the plain copy's policies
constexpr uint32_t kDefaultPackCode = 2u | 4u | (2u << 3);   // tile x1, nt loads, sc1 stores
constexpr uint32_t kDefaultUnpackCode = 2u | 4u | (3u << 3);    // tile x1, nt loads, sc1+nt stores
constexpr uint32_t kDefaultUnpackCodeOddRows = 2u | (3u << 3);  // tile x1, plain loads, sc1+nt stores
constexpr uint32_t kFlatPackCode = 128u | 4u | (2u << 3);       // flat, nt loads, sc1 stores
constexpr uint32_t kFlatUnpackCode = 128u | 4u | (1u << 3);     // flat, nt loads, nt stores
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


template <bool NT>
__device__ __forceinline__ v4u load16(gsrc_t p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

// Store with a cache policy.  The compiler only offers the non-temporal hint;
// the system-scope write-through forms (sc1) are written out as instructions.
// A store needs no wait: nothing here reads what it wrote.  The s_nop after a written-out
// store covers the one hazard the compiler cannot see through the asm: a vector-ALU write to the
// store's data registers in the next two issue slots (it handles that itself for stores it
// emits; in a loop the next instruction may well be such a write).
template <int SP>
__device__ __forceinline__ void store16(gdst_t p, v4u v) {
    if (SP == 0) *p = v;
    else if (SP == 1) __builtin_nontemporal_store(v, p);
    else if (SP == 2) asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
    else asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
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
__device__ __forceinline__ void tile_body(const CopyArgs &a, uint32_t tiles_per_unit, uint32_t align_dst,
                                          uint32_t tile_index) {
    const uint32_t u_idx = tile_index / tiles_per_unit;
    const uint32_t tile = tile_index - u_idx * tiles_per_unit;
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
    if (first >= n + lead) return;      // this tile lies beyond the descriptor's end
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
    tile_body<true, VPT, NTL, SP>(a, tiles_per_unit, align_dst, blockIdx.x);
}

template <int VPT, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_unpack_tile_kernel(const CopyArgs a, uint32_t tiles_per_unit,
                                                               uint32_t align_dst) {
    tile_body<false, VPT, NTL, SP>(a, tiles_per_unit, align_dst, blockIdx.x);
}

// Thin form of the tiled kernels: a fixed, small number of workgroups, each walking over
// the tiles gridDim.x apart.  For buffers on the far side of the host link: a few hundred
// wavefronts keep the link full (its rate times its latency is about 100 KB in flight),
// so there is no reason to fill every compute unit with wavefronts that wait for it, and
// kernels of other streams keep the machine.  The trip count is fixed at launch.
template <bool PACK, int VPT, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_tile_walk_kernel(const CopyArgs a, uint32_t tiles_per_unit,
                                                             uint32_t align_dst, uint32_t n_tiles) {
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x)
        tile_body<PACK, VPT, NTL, SP>(a, tiles_per_unit, align_dst, t);
}

// Pipelined form of the tiled kernels: a fixed grid that fills the machine once (every
// workgroup resident), each workgroup walking over the tiles gridDim.x apart with its work
// software-pipelined three deep -- while the vectors of tile i are on their way, the loads of
// tile i+1 have been issued and the descriptor of tile i+2 is being fetched.  One-shot
// workgroups (the tiled form above) start with a dependent chain, descriptor fetch then data
// load, during which their wavefronts hold a slot but have nothing in flight; on workloads of
// many small descriptors the memory system then runs below saturation (its request queues
// hardly ever push back) although every wavefront slot is taken.  Here a wavefront always has
// one or two loads outstanding and the descriptor latency is hidden behind them.  The tiles a
// workgroup visits and their order over the machine are those of the tiled form, so the
// access stream the memory sees is the same.  The trip count is fixed at launch.
struct PipeStage {
    kvl_unit_t u;       // descriptor of the stage's tile
    uint32_t tile;      // index of the tile inside its descriptor
    bool valid;         // false: the workgroup has run out of tiles
};
// The descriptors are not written while a kernel runs: read through the constant address
// space they stay scalar loads inside the loop (a plain global pointer may alias the stores
// there, and the compiler then reads it with vector loads it has to wait for at once).
typedef const kvl_unit_t __attribute__((address_space(4))) *cunits_t;

// Inside the loop nothing is conditional: a lane whose position falls outside its descriptor
// (the idle lead of an aligned first tile, the ragged end of the last) moves the descriptor's
// nearest vector instead, a duplicate of what the lane that owns that vector moves, and the
// loop covers only the trips in which every workgroup has a tile.  With a branch around a
// load or a store the compiler can no longer tell how many memory operations are in flight
// and drains them all before every store; without one it waits for exactly the load it needs.
// The last few tiles of each workgroup are done one by one after the loop.
template <bool PACK, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_tile_pipe_kernel(const CopyArgs a, uint32_t tiles_per_unit,
                                                             uint32_t align_dst, uint32_t n_tiles) {
    const uint32_t p = a.plane_begin + blockIdx.y;
    const uint32_t row = a.row_elems[p];
    const uintptr_t pool_base = a.pool[p], xfer_base = a.xfer[p];
    cunits_t units = (cunits_t)(uintptr_t)(a.units + a.unit_begin);
    const uint32_t last_unit = a.n_units - 1;               // the launcher passes at least one descriptor
    const uint32_t G = gridDim.x;                           // <= n_tiles
    // the tile `k` strides ahead of this workgroup's first is tile (k*G + blockIdx.x): kept as
    // (descriptor, tile inside it) and advanced without a division
    const uint32_t step_u = G / tiles_per_unit, step_t = G - step_u * tiles_per_unit;
    uint32_t f_u = blockIdx.x / tiles_per_unit, f_t = blockIdx.x - f_u * tiles_per_unit;   // the fetch stage's tile
    auto fetch = [&](PipeStage &s) {
        s.tile = f_t;
        s.valid = f_u <= last_unit;
        cunits_t q = units + (f_u <= last_unit ? f_u : last_unit);     // always a load, never past the end
        s.u.pool_row = q->pool_row;
        s.u.xfer_row = q->xfer_row;
        s.u.n_rows = q->n_rows;
        f_u += step_u;
        f_t += step_t;
        if (f_t >= tiles_per_unit) {
            f_t -= tiles_per_unit;
            ++f_u;
        }
    };
    // this lane's vector of a stage's tile (descriptors are never empty)
    auto place = [&](const PipeStage &s, gsrc_t &src, gdst_t &dst) {
        const uint32_t n = s.u.n_rows * row;
        const uintptr_t pool = pool_base + (uint64_t)s.u.pool_row * row * 16u;
        const uintptr_t xfer = xfer_base + (uint64_t)s.u.xfer_row * row * 16u;
        const uint32_t lead = align_dst ? ((uint32_t)((PACK ? xfer : pool) >> 4) & 7u) : 0u;
        const uint32_t pos = s.tile * blockDim.x + threadIdx.x;
        uint32_t j = pos >= lead ? pos - lead : 0u;
        j = j < n ? j : n - 1;
        src = (gsrc_t)(PACK ? pool : xfer) + j;
        dst = (gdst_t)(PACK ? xfer : pool) + j;
    };
    // trips in which every workgroup has a tile; the loop takes them two at a time and stops
    // two short, so that its three stages never run past them
    const uint32_t full = n_tiles / G;
    const uint32_t looped = full >= 2 ? (full - 2) & ~1u : 0u;
    // Two sets of registers, A for the even tiles and B for the odd ones, so that nothing is
    // moved from one to the other (a move of loaded data would have to wait for it).
    PipeStage s_a, s_b;
    gsrc_t src_a, src_b;
    gdst_t dst_a, dst_b;
    v4u v_a, v_b;
    fetch(s_a);                                   // tile 0 of this workgroup (there always is one)
    fetch(s_b);                                   // tile 1
    place(s_a, src_a, dst_a);
    v_a = load16<NTL>(src_a);
    fetch(s_a);                                   // tile 2
    for (uint32_t i = 0; i < looped; i += 2) {
        // (a scalar load can only be waited for together with every other one in flight, so a
        // descriptor is fetched after the step's use of the one fetched before it)
        place(s_b, src_b, dst_b);
        v_b = load16<NTL>(src_b);                 // tile i + 1 on its way
        fetch(s_b);                               // descriptor of tile i + 3, first needed two steps on
        store16<SP>(dst_a, v_a);                  // tile i: waits for its own load only
        place(s_a, src_a, dst_a);
        v_a = load16<NTL>(src_a);                 // tile i + 2
        fetch(s_a);                               // tile i + 4
        store16<SP>(dst_b, v_b);                  // tile i + 1
    }
    // in flight: tile `looped` in v_a; s_b holds tile looped + 1, s_a tile looped + 2
    store16<SP>(dst_a, v_a);
    // the remaining tiles of this workgroup (at most three: looped + 1, + 2, + 3), one at a
    // time; they may not exist, and their idle lanes are switched off rather than duplicated
    PipeStage s_c;
    fetch(s_c);                                   // tile looped + 3
    auto copy_tile = [&](const PipeStage &s) {
        const uint32_t n = s.valid ? s.u.n_rows * row : 0u;
        const uintptr_t pool = pool_base + (uint64_t)s.u.pool_row * row * 16u;
        const uintptr_t xfer = xfer_base + (uint64_t)s.u.xfer_row * row * 16u;
        const uint32_t lead = align_dst ? ((uint32_t)((PACK ? xfer : pool) >> 4) & 7u) : 0u;
        const uint32_t pos = s.tile * blockDim.x + threadIdx.x;
        if (pos >= lead && pos - lead < n) {
            gsrc_t sp = (gsrc_t)(PACK ? pool : xfer) + (pos - lead);
            gdst_t dp = (gdst_t)(PACK ? xfer : pool) + (pos - lead);
            store16<SP>(dp, load16<NTL>(sp));
        }
    };
    copy_tile(s_b);
    copy_tile(s_a);
    copy_tile(s_c);
}

// Flat form for descriptors much smaller than a workgroup: the lanes of the launch are
// dealt to the descriptors m at a time (m = max_unit_rows * row, the vectors of the
// largest descriptor), so lane g moves vector g mod m of descriptor g div m; a shorter
// descriptor leaves its last lanes idle.  Every lane reads its own descriptor (lanes of
// one descriptor read the same 16 bytes).  The launcher keeps n_units * m below 2^32.
template <bool PACK, bool NTL, int SP>
__global__ void __launch_bounds__(1024) kvl_flat_kernel(const CopyArgs a, uint32_t max_unit_rows) {
    const uint32_t p = a.plane_begin + blockIdx.y;
    const uint32_t row = a.row_elems[p];
    const uint32_t m = max_unit_rows * row;
    const uint32_t g = blockIdx.x * blockDim.x + threadIdx.x;
    const uint32_t u_idx = g / m;
    if (u_idx >= a.n_units) return;
    const uint32_t off = g - u_idx * m;
    const kvl_unit_t u = a.units[a.unit_begin + u_idx];
    if (off >= u.n_rows * row) return;
    gsrc_t src = (gsrc_t)((PACK ? a.pool[p] : a.xfer[p]) + (uint64_t)(PACK ? u.pool_row : u.xfer_row) * row * 16u);
    gdst_t dst = (gdst_t)((PACK ? a.xfer[p] : a.pool[p]) + (uint64_t)(PACK ? u.xfer_row : u.pool_row) * row * 16u);
    store16<SP>(dst + off, load16<NTL>(src + off));
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

// A tile is VPT * blockDim elements of a descriptor; lane t takes elements t, t + blockDim, ...
// of it, all loads before the first store.
template <bool TO_POOL, bool VEC, int VPT>
__device__ __forceinline__ void fullblock_tile(const FullBlockArgs &a, uint32_t tiles_per_unit, uint32_t tile_index) {
    const uint32_t u_idx = tile_index / tiles_per_unit;
    const uint32_t tile = tile_index - u_idx * tiles_per_unit;
    const kvl_unit_t u = a.units[u_idx];
    const uint32_t p = blockIdx.y;
    const uint32_t row = a.row_elems[p];
    const uint32_t n = u.n_rows * row;
    const uint32_t first = tile * (blockDim.x * VPT) + threadIdx.x;
    if (first >= n) return;
    const uint32_t within = u.pool_row % a.block_tokens;
    const uint64_t in_pool = (uint64_t)u.pool_row * row;
    const uint64_t in_blocks = (uint64_t)u.block_index * a.fb_elems + a.layer_plane_off[p] + (uint64_t)within * row;
    if (VEC) {
        gsrc_t src = TO_POOL ? (gsrc_t)a.blocks + in_blocks : (gsrc_t)a.pool[p] + in_pool;
        gdst_t dst = TO_POOL ? (gdst_t)a.pool[p] + in_pool : (gdst_t)a.blocks + in_blocks;
        v4u v[VPT];
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t i = first + k * blockDim.x;
            if (i < n) v[k] = TO_POOL ? load16<false>(src + i) : load16<true>(src + i);
        }
#pragma unroll
        for (int k = 0; k < VPT; ++k) {
            const uint32_t i = first + k * blockDim.x;
            if (i < n) {
                if (TO_POOL) store16<3>(dst + i, v[k]);
                else store16<0>(dst + i, v[k]);
            }
        }
    } else {
        uint8_t *pool = reinterpret_cast<uint8_t *>(a.pool[p]) + in_pool;
        uint8_t *blocks = reinterpret_cast<uint8_t *>(a.blocks) + in_blocks;
        for (int k = 0; k < VPT; ++k) {
            const uint32_t i = first + k * blockDim.x;
            if (i >= n) break;
            if (TO_POOL) pool[i] = blocks[i];
            else blocks[i] = pool[i];
        }
    }
}

// gridDim.x workgroups walk over the n_tiles tiles (one tile each when there are as many).
template <bool TO_POOL, bool VEC, int VPT>
__global__ void __launch_bounds__(256) kvl_fullblock_kernel(const FullBlockArgs a, uint32_t tiles_per_unit,
                                                            uint32_t n_tiles) {
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x)
        fullblock_tile<TO_POOL, VEC, VPT>(a, tiles_per_unit, t);
}

// Reference streams for measuring what the memory can do (kvl_ceiling_kernel): the tiled form
// with its addresses computed instead of read from descriptors.  Block u of the dense side
// lives in block (u * mul) mod 2^k of the hopping side (mul odd: a bijection), or in block
// table[u] if a table is given (one scalar load, as the descriptor fetch of the real kernels).
struct CeilingArgs {
    uintptr_t dense, hopping;       // base addresses
    const uint32_t *table;          // optional
    uint64_t tile_magic;            // ceil(2^40 / tiles_per_block): block of a workgroup by multiplication
    uint32_t n_blocks, hop_mask, mul;
    uint32_t block_vecs, tiles_per_block, skew_vecs, n_vecs;
};

// MODE 0: copy, 1: read only, 2: write only.  GATHER: the source hops, else the destination.
template <int MODE, bool GATHER, bool NTL, int SP>
__global__ void __launch_bounds__(256) kvl_ceiling_pattern_kernel(const CeilingArgs a) {
    const uint32_t w = blockIdx.x;
    const uint32_t u = (uint32_t)(((uint64_t)w * a.tile_magic) >> 40);
    const uint32_t tile = w - u * a.tiles_per_block;
    const uint32_t hb = a.table ? a.table[u] : ((u * a.mul) & a.hop_mask);
    const uintptr_t hop = a.hopping + (uint64_t)hb * a.block_vecs * 16u;
    const uintptr_t den = a.dense + ((uint64_t)u * a.block_vecs + a.skew_vecs) * 16u;
    gsrc_t src = (gsrc_t)(GATHER ? hop : den);
    gdst_t dst = (gdst_t)(GATHER ? den : hop);
    const uint32_t lead = (uint32_t)((GATHER ? den : hop) >> 4) & 7u;     // tiles start on a destination line
    const uint32_t pos = tile * blockDim.x + threadIdx.x;
    if (pos < lead || pos - lead >= a.block_vecs) return;
    if (MODE == 0) {
        store16<SP>(dst + (pos - lead), load16<NTL>(src + (pos - lead)));
    } else if (MODE == 1) {
        const v4u v = load16<NTL>(src + (pos - lead));
        if (v.x == 0x9e3779b9u && v.y == 0x7f4a7c15u && v.z == 0xf39cc060u && v.w == 0x5cedc834u)
            store16<SP>(dst + (pos - lead), v);     // keeps the load alive; the pattern does not occur in the buffers
    } else {
        const v4u v = {pos, u, tile, hb};
        store16<SP>(dst + (pos - lead), v);
    }
}

template <int MODE, bool NTL, int SP>
__global__ void __launch_bounds__(256) kvl_ceiling_linear_kernel(const v4u *src, v4u *dst, uint64_t n) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (MODE == 0) {
        store16<SP>((gdst_t)dst + i, load16<NTL>((gsrc_t)src + i));
    } else if (MODE == 1) {
        const v4u v = load16<NTL>((gsrc_t)src + i);
        if (v.x == 0x9e3779b9u && v.y == 0x7f4a7c15u && v.z == 0xf39cc060u && v.w == 0x5cedc834u)
            store16<SP>((gdst_t)dst + i, v);
    } else {
        const v4u v = {(uint32_t)i, 1u, 2u, 3u};
        store16<SP>((gdst_t)dst + i, v);
    }
}

// Straight copy, one vector per lane: the tiled kernel without descriptors.
__global__ void __launch_bounds__(256) kvl_linear_kernel(const v4u *src, v4u *dst, uint64_t n) {
    const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) store16<kLinearStorePolicy>((gdst_t)dst + i, load16<kLinearNtLoad>((gsrc_t)src + i));
}

}  // namespace kvl
