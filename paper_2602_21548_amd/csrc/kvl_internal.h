// Internal declarations shared by the library's translation units.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

#include "kvl.h"

struct kvl_plan_s {
    kvl_layout_t layout{};
    uint32_t flags = 0;
    bool paired = false;                         // made by kvl_plan_pair: xfer_row holds destination pool rows
    uint64_t dst_pool_blocks = 0;                // paired plans: blocks of the destination pool
    uint32_t n_req = 0;
    uint64_t hit_tokens = 0;                     // T
    uint64_t payload_bytes = 0;                  // all planes
    uint64_t plane_base[KVL_MAX_PLANES] = {};    // byte offset of each plane in the transfer buffer
    uint32_t max_unit_rows = 0;
    uint64_t blocks_touched = 0;                 // Full Blocks a buffer of this plan's ranges holds
    bool vec16 = false;                          // every row size is a multiple of 16 bytes
    std::vector<kvl_unit_t> units;               // host copy of the descriptors
    bool threads_chosen = false;                 // the caller named block_threads (else the launcher may halve the default)
    std::vector<uint32_t> block_first_unit;      // KVL_NO_MERGE plans, made on demand: first descriptor of each block
    std::vector<uint32_t> block_row_lo, block_row_hi;   // with it: rows [lo, hi) of each block that the plan moves
    kvl_unit_t *d_units = nullptr;               // device copy (absent for KVL_HOST_ONLY)
    size_t d_units_capacity = 0;                 // bytes of the cached buffer d_units lives in
    int device = -1;
    // One event per stream on which kernels that read d_units were enqueued (the caller's streams and
    // the lanes), re-recorded after every such launch: once all of them have fired no kernel reads the
    // buffer any more and it may be handed to another plan.  Recorded at launch time because a stream
    // of the caller's may be gone by the time the plan is destroyed.
    mutable std::vector<std::pair<hipStream_t, hipEvent_t>> stream_events;
    mutable bool untracked_use = false;          // a launch could not be followed (too many streams, a stream
                                                 // under capture, a failed record): wait for the device instead
    kvl_tuning_t tuning{};                       // resolved (no zero fields)
    // h2d path: one lane (a stream of the library's own) and one "lane done" event per staging slot
    std::vector<hipStream_t> lanes;
    std::vector<uint32_t> lane_cu_mask;          // empty: lanes may use every compute unit
    std::vector<hipEvent_t> ev_lane_done;
    hipEvent_t ev_entry = nullptr, ev_entry2 = nullptr;
};

namespace kvl {

void set_hip_error(hipError_t e);

#define KVL_HIP(expr)                                   \
    do {                                                \
        hipError_t kvl_e_ = (expr);                     \
        if (kvl_e_ != hipSuccess) {                     \
            ::kvl::set_hip_error(kvl_e_);               \
            return KVL_EHIP;                            \
        }                                               \
    } while (0)

constexpr uint32_t kDefaultUnitBytes = 128u << 10;
constexpr uint32_t kDefaultBlockThreads = 256;
constexpr uint32_t kHostSideGroups = 64;    // workgroups of a kernel whose far side is host memory (see kvl_tile_walk_kernel)
constexpr uint32_t kNumVariants = 512;       // explicit variants are 1 .. kNumVariants
bool valid_block_threads(uint32_t t);

// A launch may not have 2^32 or more lanes along x.  How many workgroups of `threads` lanes a
// launch over `work` workgroups' worth of tiles gets: all of them if that fits (and no cap is
// asked for), else as many as fit, each walking over several tiles.  *walk says which.
constexpr uint64_t kMaxLanesPerLaunch = (1ull << 32) - 1;
inline uint32_t launch_groups(uint64_t work, uint32_t threads, uint32_t cap, bool *walk) {
    uint64_t most = kMaxLanesPerLaunch / threads;
    if (cap && cap < most) most = cap;
    *walk = work > most;
    return (uint32_t)(*walk ? most : work);
}

// Cut [0, n_units) of one plane into chunks of at most chunk_bytes.
int make_chunks(const kvl_plan_t *plan, uint64_t chunk_bytes, std::vector<kvl_chunk_t> &out);

// Enqueue the copy of descriptors [unit_begin, unit_end) of planes
// [plane_begin, plane_end).  xfer_plane[p] is the address at which transfer row
// 0 of plane p would lie (it may point before a staging slot; only rows of the
// given descriptors are touched).
// far_host: the transfer side lies in host memory (the kernel crosses the host link).
int launch_units(const kvl_plan_t *plan, bool pack, uint32_t unit_begin, uint32_t unit_end,
                 uint32_t plane_begin, uint32_t plane_end,
                 void *const *pool_planes, const uintptr_t *xfer_plane, hipStream_t stream,
                 bool far_host = false);
// true if HIP knows ptr as pinned host memory (false when the plan skips pointer checks)
bool is_host_memory(const kvl_plan_t *plan, const void *ptr);

int upload_units(kvl_plan_t *plan);
// a kernel reading the plan's descriptors has just been enqueued on `stream`
void mark_launch(const kvl_plan_t *plan, hipStream_t stream);
void drop_stream_events(const kvl_plan_t *plan);
// lanes come from, and go back to, a small pool shared by all plans
hipStream_t take_pooled_lane(int device);
void return_lane(hipStream_t lane, int device);
// kvl_check_buffer unless the plan opted out
int check_buffer(const kvl_plan_t *plan, const void *ptr, uint64_t bytes, bool allow_host);
int check_pool(const kvl_plan_t *plan, const void *const *planes, uint64_t pool_blocks);
int ensure_lanes(kvl_plan_t *plan, size_t lanes);
int lanes_follow(kvl_plan_t *plan, size_t lanes, hipStream_t copy_s, hipStream_t kern_s);

int check_device(const kvl_plan_t *plan);
uint64_t layer_block_bytes(const kvl_plan_t *plan);
int check_fullblock_args(const kvl_plan_t *plan, bool to_pool, uint64_t blocks_bytes, uint32_t layer);
int fullblock_launch(const kvl_plan_t *plan, bool to_pool, uintptr_t base, uint64_t block_pitch,
                     uint64_t layer_off, uint32_t unit_begin, uint32_t unit_end,
                     void *const *pool_planes, hipStream_t stream, bool far_host = false);
// Enqueue the move of one layer between a buffer of Full Blocks and a paged pool.
int fullblock_layer(const kvl_plan_t *plan, bool to_pool, uintptr_t blocks, uint64_t blocks_bytes,
                    uint32_t layer, void *const *pool_planes, hipStream_t stream);


// Host-buffer paths (kvl_h2d.hip), shared with the layer-wise streaming loop.
int enqueue_h2d_layer(kvl_plan_t *plan, const std::vector<kvl_chunk_t> &chunks,
                      const void *host_xfer, void *dev_staging, uint64_t chunk_bytes, size_t lanes,
                      void *const *pool_planes, hipStream_t kern_s, hipEvent_t wait_before_scatter);
int check_h2d_args(const kvl_plan_t *plan, const void *host, const void *staging,
                   uint64_t staging_bytes, uint64_t chunk_bytes, size_t *slots);
int enqueue_zero_copy_layer(const kvl_plan_t *plan, const void *host_xfer, void *const *pool_planes,
                            hipStream_t kern_s, hipEvent_t wait_before_scatter);
int enqueue_d2h_pack_layer(kvl_plan_t *plan, const std::vector<kvl_chunk_t> &chunks,
                           const void *const *pool_planes, void *dev_staging, uint64_t chunk_bytes,
                           size_t lanes, void *host_xfer, hipEvent_t wait_first, hipStream_t collector);
int check_d2h_args(const kvl_plan_t *plan, const void *staging, uint64_t staging_bytes, uint64_t chunk_bytes,
                   const void *host, uint64_t host_capacity, size_t *slots);
int check_fullblock_staging(const kvl_plan_t *plan, const void *staging, uint64_t staging_bytes,
                            uint64_t chunk_bytes, size_t *slots);
int enqueue_h2d_fullblocks_layer(kvl_plan_t *plan, const void *full_blocks, uint32_t layer,
                                 void *dev_staging, uint64_t chunk_bytes, size_t lanes,
                                 void *const *pool_planes, hipStream_t kern_s, hipEvent_t wait_before_scatter);

}  // namespace kvl
