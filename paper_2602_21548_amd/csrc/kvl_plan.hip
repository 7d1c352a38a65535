// Host side of the library: batch validation, transfer-buffer layout and copy
// descriptors (kvl_plan), plan inspection, error text.
#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>

#include "kvl_internal.h"

namespace kvl {

static thread_local hipError_t g_last_hip = hipSuccess;

void set_hip_error(hipError_t e) { g_last_hip = e; }

bool valid_block_threads(uint32_t t) {
    return t == 64 || t == 128 || t == 256 || t == 512 || t == 1024;
}

int make_chunks(const kvl_plan_t *plan, uint64_t chunk_bytes, std::vector<kvl_chunk_t> &out) {
    out.clear();
    if (chunk_bytes == 0) return KVL_EINVAL;
    const auto &u = plan->units;
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p) {
        const uint64_t row = plan->layout.row_bytes[p];
        if ((uint64_t)plan->max_unit_rows * row > chunk_bytes) return KVL_ESPACE;
        size_t i = 0;
        while (i < u.size()) {
            kvl_chunk_t c{};
            c.plane = p;
            c.unit_begin = (uint32_t)i;
            c.host_offset = plan->plane_base[p] + (uint64_t)u[i].xfer_row * row;
            uint64_t bytes = 0;
            while (i < u.size() && bytes + (uint64_t)u[i].n_rows * row <= chunk_bytes) {
                bytes += (uint64_t)u[i].n_rows * row;
                ++i;
            }
            c.unit_end = (uint32_t)i;
            c.bytes = bytes;
            out.push_back(c);
        }
    }
    return KVL_OK;
}

// Descriptor arrays come from a small per-process cache, so that a caller who builds a plan
// per batch pays neither a device allocation nor a device free (both synchronise the device,
// and a free can stall the next launch for tens of milliseconds).  A destroyed plan's array is
// retired, not freed: every launch that reads it is followed by an event on its stream (one event
// per stream, recorded again after each launch), and the array goes back to the cache only when
// those events have fired.  Nothing here waits for the device; only kvl_release_cached_memory
// blocks (on the retired arrays' own events).
namespace {
struct CachedBuffer {
    void *ptr;
    size_t capacity;
    int device;
};
struct RetiredBuffer {
    CachedBuffer buf;
    std::vector<hipEvent_t> events;     // all fired: no kernel reads the buffer any more
};
struct PooledLane {
    hipStream_t stream;
    int device;
};
std::mutex g_cache_mutex;               // guards everything below
std::vector<CachedBuffer> g_cache;
std::vector<RetiredBuffer> g_retired;
std::vector<std::pair<hipEvent_t, int>> g_events;       // spare events, with their device
std::vector<PooledLane> g_lanes;
constexpr size_t kCacheEntries = 16;
constexpr size_t kCacheBytes = 256u << 20;      // never keep more than this much idle
constexpr size_t kSpareEvents = 256;
constexpr size_t kPooledLanes = 16;
constexpr size_t kTrackedStreams = 24;

size_t round_capacity(size_t bytes) {
    size_t cap = 64u << 10;
    while (cap < bytes) cap <<= 1;
    return cap;
}

// with g_cache_mutex held and `device` current
hipEvent_t take_event(int device) {
    for (size_t i = 0; i < g_events.size(); ++i) {
        if (g_events[i].second == device) {
            hipEvent_t e = g_events[i].first;
            g_events.erase(g_events.begin() + (long)i);
            return e;
        }
    }
    // The events only say "the kernels before this point have finished": no timing, and no
    // system-scope cache flush when they fire (nothing is read back through them).
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming | hipEventDisableSystemFence) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    return e;
}

void give_event(hipEvent_t e, int device) {
    if (g_events.size() < kSpareEvents) {
        try {
            g_events.emplace_back(e, device);
            return;
        } catch (const std::bad_alloc &) {
        }
    }
    (void)hipEventDestroy(e);
}

// a buffer nobody reads any more: keep it for the next plan, or free it if the cache is full
void keep_or_free(const CachedBuffer &b) {
    size_t held = 0;
    for (const CachedBuffer &c : g_cache) held += c.capacity;
    if (g_cache.size() < kCacheEntries && held + b.capacity <= kCacheBytes) {
        try {
            g_cache.push_back(b);
            return;
        } catch (const std::bad_alloc &) {
        }
    }
    (void)hipFree(b.ptr);
}

// move the retired buffers whose events have all fired to the cache; `wait`: block for them
void reap_retired(bool wait) {
    for (size_t i = 0; i < g_retired.size();) {
        RetiredBuffer &r = g_retired[i];
        bool done = true;
        for (hipEvent_t e : r.events) {
            const hipError_t q = wait ? hipEventSynchronize(e) : hipEventQuery(e);
            if (q == hipErrorNotReady) {
                done = false;
                break;
            }
            if (q != hipSuccess) (void)hipGetLastError();       // a broken event cannot hold the buffer for ever
        }
        if (!done) {
            ++i;
            continue;
        }
        for (hipEvent_t e : r.events) give_event(e, r.buf.device);
        keep_or_free(r.buf);
        g_retired.erase(g_retired.begin() + (long)i);
    }
}
}  // namespace

void mark_launch(const kvl_plan_t *plan, hipStream_t stream) {
    if (plan->flags & KVL_CALLER_SYNCS) return;            // the caller answers for the plan's lifetime
    // a launch that is being captured into a graph runs whenever the graph is replayed: not ours to follow
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) {
        (void)hipGetLastError();
        plan->untracked_use = true;
        return;
    }
    if (capture != hipStreamCaptureStatusNone) {
        plan->untracked_use = true;
        return;
    }
    hipEvent_t ev = nullptr;
    for (const auto &se : plan->stream_events)
        if (se.first == stream) ev = se.second;
    if (!ev) {
        if (plan->stream_events.size() >= kTrackedStreams) {
            plan->untracked_use = true;
            return;
        }
        {
            std::lock_guard<std::mutex> lock(g_cache_mutex);
            ev = take_event(plan->device);
        }
        if (!ev) {
            plan->untracked_use = true;
            return;
        }
        try {
            plan->stream_events.emplace_back(stream, ev);
        } catch (const std::bad_alloc &) {
            std::lock_guard<std::mutex> lock(g_cache_mutex);
            give_event(ev, plan->device);
            plan->untracked_use = true;
            return;
        }
    }
    if (hipEventRecord(ev, stream) != hipSuccess) {
        (void)hipGetLastError();
        plan->untracked_use = true;
    }
}

void drop_stream_events(const kvl_plan_t *plan) {
    if (plan->stream_events.empty()) return;
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    for (const auto &se : plan->stream_events) give_event(se.second, plan->device);
    plan->stream_events.clear();
}

hipStream_t take_pooled_lane(int device) {
    std::lock_guard<std::mutex> lock(g_cache_mutex);
    for (size_t i = 0; i < g_lanes.size(); ++i) {
        if (g_lanes[i].device == device) {
            hipStream_t s = g_lanes[i].stream;
            g_lanes.erase(g_lanes.begin() + (long)i);
            return s;
        }
    }
    return nullptr;
}

// A lane that is not needed any more; work may still be queued on it (it runs to its end there:
// a lane is an in-order stream, and whoever takes it from the pool queues behind that work).
void return_lane(hipStream_t lane, int device) {
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        if (g_lanes.size() < kPooledLanes) {
            try {
                g_lanes.push_back(PooledLane{lane, device});
                return;
            } catch (const std::bad_alloc &) {
            }
        }
    }
    (void)hipStreamSynchronize(lane);
    (void)hipStreamDestroy(lane);
}

static hipError_t descriptor_alloc(void **out, size_t bytes, size_t *capacity, int device) {
    const size_t want = round_capacity(bytes);
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        reap_retired(false);
        for (size_t i = 0; i < g_cache.size(); ++i) {
            if (g_cache[i].device == device && g_cache[i].capacity == want) {
                *out = g_cache[i].ptr;
                *capacity = want;
                g_cache.erase(g_cache.begin() + (long)i);
                return hipSuccess;
            }
        }
    }
    *capacity = want;
    return hipMalloc(out, want);
}

// The plan is going away: its descriptor array may be reused once the events recorded after its
// launches have fired.  No stream is touched here.
static void descriptor_release(const kvl_plan_t *plan) {
    RetiredBuffer r{CachedBuffer{plan->d_units, plan->d_units_capacity, plan->device}, {}};
    if (plan->flags & KVL_CALLER_SYNCS) {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        keep_or_free(r.buf);
        return;
    }
    bool tracked = !plan->untracked_use;
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        if (tracked) {
            try {
                for (const auto &se : plan->stream_events) r.events.push_back(se.second);
                g_retired.push_back(std::move(r));
                r.buf.ptr = nullptr;
            } catch (const std::bad_alloc &) {
                tracked = false;
            }
        }
        if (r.buf.ptr)
            for (const auto &se : plan->stream_events) give_event(se.second, plan->device);
    }
    plan->stream_events.clear();
    if (r.buf.ptr) {
        // some launch could not be followed: fall back to what a device free would have done
        int current = plan->device;
        (void)hipGetDevice(&current);
        if (current != plan->device) (void)hipSetDevice(plan->device);
        (void)hipDeviceSynchronize();
        if (current != plan->device) (void)hipSetDevice(current);
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        keep_or_free(r.buf);
    }
}

int check_buffer(const kvl_plan_t *plan, const void *ptr, uint64_t bytes, bool allow_host) {
    if (plan->flags & KVL_NO_POINTER_CHECKS) return KVL_OK;
    return kvl_check_buffer(ptr, bytes, allow_host ? 1 : 0);
}

bool is_host_memory(const kvl_plan_t *plan, const void *ptr) {
    if (!ptr || (plan->flags & KVL_NO_POINTER_CHECKS)) return false;
    hipPointerAttribute_t a{};
    if (hipPointerGetAttributes(&a, ptr) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return a.type == hipMemoryTypeHost;
}

// Descriptors go up on a stream of the library's own, out of pinned memory, and the call waits
// for that copy alone: a plain hipMemcpy would also wait for whatever the caller has running on
// the default stream.
namespace {
struct Uploader {
    hipStream_t stream = nullptr;
    void *bounce = nullptr;         // pinned
    size_t capacity = 0;
};
std::mutex g_upload_mutex;
Uploader g_uploaders[64];
constexpr size_t kBounceLimit = 64u << 20;      // larger descriptor arrays are copied from pageable memory
}  // namespace

int upload_units(kvl_plan_t *plan) {
    hipError_t e = hipGetDevice(&plan->device);
    if (e == hipSuccess && !plan->units.empty()) {
        const size_t bytes = plan->units.size() * sizeof(kvl_unit_t);
        e = descriptor_alloc((void **)&plan->d_units, bytes, &plan->d_units_capacity, plan->device);
        if (e == hipSuccess && plan->device >= 0 && plan->device < 64) {
            std::lock_guard<std::mutex> lock(g_upload_mutex);
            Uploader &u = g_uploaders[plan->device];
            if (!u.stream) e = hipStreamCreateWithFlags(&u.stream, hipStreamNonBlocking);
            if (e == hipSuccess && bytes <= kBounceLimit && u.capacity < bytes) {
                if (u.bounce) (void)hipHostFree(u.bounce);
                u.bounce = nullptr;
                u.capacity = 0;
                size_t cap = 1u << 20;
                while (cap < bytes) cap <<= 1;
                if (hipHostMalloc(&u.bounce, cap, hipHostMallocDefault) == hipSuccess) u.capacity = cap;
                else (void)hipGetLastError();       // no pinned memory to be had: copy from where the descriptors are
            }
            if (e == hipSuccess) {
                const void *from = plan->units.data();
                if (u.capacity >= bytes) {
                    std::memcpy(u.bounce, plan->units.data(), bytes);
                    from = u.bounce;
                }
                e = hipMemcpyAsync(plan->d_units, from, bytes, hipMemcpyHostToDevice, u.stream);
                if (e == hipSuccess) e = hipStreamSynchronize(u.stream);
            }
        } else if (e == hipSuccess) {
            e = hipMemcpy(plan->d_units, plan->units.data(), bytes, hipMemcpyHostToDevice);
        }
    }
    if (e != hipSuccess) {
        set_hip_error(e);
        return KVL_EHIP;
    }
    return KVL_OK;
}

static int resolve_tuning(const kvl_tuning_t *in, kvl_tuning_t *out) {
    kvl_tuning_t t{};
    if (in) t = *in;
    if (t.unit_bytes == 0) t.unit_bytes = kDefaultUnitBytes;
    if (t.block_threads == 0) t.block_threads = kDefaultBlockThreads;
    if (!valid_block_threads(t.block_threads)) return KVL_EINVAL;
    if (t.variant > kNumVariants) return KVL_EINVAL;
    if (t.unit_bytes > (1u << 30)) t.unit_bytes = 1u << 30;
    *out = t;
    return KVL_OK;
}

static int build(const kvl_layout_t *layout, const kvl_request_t *req, uint32_t n_req,
                 uint32_t flags, const kvl_tuning_t *tuning, kvl_plan_t **out) {
    if (!layout || !out || (n_req && !req)) return KVL_EINVAL;
    *out = nullptr;
    if (!(flags & (KVL_GATHER | KVL_SCATTER))) return KVL_EINVAL;
    if (flags & ~(KVL_GATHER | KVL_SCATTER | KVL_HOST_ONLY | KVL_NO_MERGE | KVL_TOKENS_APPEND | KVL_TOKENS_ALL |
                  KVL_NO_POINTER_CHECKS | KVL_CALLER_SYNCS))
        return KVL_EINVAL;
    if ((flags & KVL_TOKENS_APPEND) && (flags & KVL_TOKENS_ALL)) return KVL_EINVAL;
    if (layout->block_tokens == 0 || layout->n_planes == 0 || layout->n_planes > KVL_MAX_PLANES)
        return KVL_EINVAL;
    const uint64_t bs = layout->block_tokens;
    uint32_t max_row = 0;
    bool vec16 = true;
    for (uint32_t p = 0; p < layout->n_planes; ++p) {
        if (layout->row_bytes[p] == 0) return KVL_EINVAL;
        max_row = std::max(max_row, layout->row_bytes[p]);
        vec16 = vec16 && (layout->row_bytes[p] % 16 == 0);
    }
    // descriptors index token rows with 32 bits
    if (layout->pool_blocks > UINT32_MAX / bs) return KVL_ERANGE;

    kvl_plan_t *plan = new (std::nothrow) kvl_plan_t;
    if (!plan) return KVL_ENOMEM;
    plan->layout = *layout;
    for (uint32_t p = layout->n_planes; p < KVL_MAX_PLANES; ++p) plan->layout.row_bytes[p] = 0;
    plan->flags = flags;
    plan->n_req = n_req;
    plan->vec16 = vec16;
    int rc = resolve_tuning(tuning, &plan->tuning);
    if (rc != KVL_OK) { delete plan; return rc; }
    plan->threads_chosen = tuning && tuning->block_threads != 0;

    const uint64_t max_rows = std::max<uint64_t>(1, plan->tuning.unit_bytes / max_row);
    const bool scatter = (flags & KVL_SCATTER) != 0;
    const bool merge = !(flags & KVL_NO_MERGE);

    try {
        // which destination blocks a scatter plan has named already: one array per thread, kept
        // from plan to plan; an entry counts only if it carries this plan's stamp, so nothing is
        // cleared between plans
        static thread_local std::vector<uint32_t> taken;
        static thread_local uint32_t stamp = 0;
        if (scatter) {
            if (taken.size() < layout->pool_blocks) taken.resize((size_t)layout->pool_blocks, 0);
            if (++stamp == 0) {                     // the stamps have wrapped: start over
                std::fill(taken.begin(), taken.end(), 0u);
                stamp = 1;
            }
        }

        // token range of request q that this plan moves
        auto range = [flags](const kvl_request_t &q, uint64_t *t0, uint64_t *t1) {
            if (flags & KVL_TOKENS_APPEND) {
                *t0 = q.hit_tokens;
                *t1 = (uint64_t)q.hit_tokens + q.append_tokens;
            } else if (flags & KVL_TOKENS_ALL) {
                *t0 = 0;
                *t1 = (uint64_t)q.hit_tokens + q.append_tokens;
            } else {
                *t0 = 0;
                *t1 = q.hit_tokens;
            }
        };
        uint64_t T = 0, touched = 0;
        for (uint32_t r = 0; r < n_req; ++r) {
            uint64_t t0, t1;
            range(req[r], &t0, &t1);
            T += t1 - t0;
            if (t1 > t0) touched += (t1 + bs - 1) / bs - t0 / bs;
        }
        if (T > UINT32_MAX) { delete plan; return KVL_ERANGE; }
        plan->hit_tokens = T;

        // First the runs: maximal spans of token rows that are contiguous on both sides (a block,
        // or physically adjacent blocks of one request merged).  run.block_index is the touched
        // block of the run's first row (whose row inside that block is pool_row mod block_tokens).
        std::vector<kvl_unit_t> runs;
        runs.reserve((size_t)std::min<uint64_t>(touched, (uint64_t)INT32_MAX));
        uint64_t xfer_row = 0;
        uint64_t block_base = 0;          // touched blocks of the requests before r
        for (uint32_t r = 0; r < n_req; ++r) {
            const kvl_request_t &q = req[r];
            const uint64_t tokens = (uint64_t)q.hit_tokens + q.append_tokens;
            const uint64_t need = (tokens + bs - 1) / bs;
            if (q.n_blocks < need) { delete plan; return KVL_ERANGE; }
            if (need && !q.block_table) { delete plan; return KVL_EINVAL; }
            for (uint64_t b = 0; b < need; ++b) {
                const int64_t id = q.block_table[b];
                if (id < 0 || (uint64_t)id >= layout->pool_blocks) { delete plan; return KVL_ERANGE; }
            }
            uint64_t t0, t1;
            range(q, &t0, &t1);
            if (t1 == t0) continue;
            const uint64_t b_first = t0 / bs, b_end = (t1 + bs - 1) / bs;   // blocks [b_first, b_end) are touched
            if (scatter) {
                for (uint64_t b = b_first; b < b_end; ++b) {
                    uint32_t &t = taken[(size_t)q.block_table[b]];
                    if (t == stamp) { delete plan; return KVL_EALIAS; }
                    t = stamp;
                }
            }
            // rows of block b that lie in the range: [lo, hi) in request tokens
            auto lo_of = [&](uint64_t b) { return std::max<uint64_t>(t0, b * bs); };
            auto hi_of = [&](uint64_t b) { return std::min<uint64_t>(t1, (b + 1) * bs); };
            // walk the touched blocks, growing a run while it ends on a block
            // boundary and the next block is the physical successor
            uint64_t b = b_first;
            while (b < b_end) {
                const uint64_t first = (uint64_t)q.block_table[b];
                const uint64_t within = lo_of(b) - b * bs;
                uint64_t rows = hi_of(b) - lo_of(b);
                uint64_t e = b + 1;
                while (merge && e < b_end && hi_of(e - 1) == e * bs &&
                       (uint64_t)q.block_table[e] == first + (e - b)) {
                    rows += hi_of(e) - lo_of(e);
                    ++e;
                }
                runs.push_back(kvl_unit_t{(uint32_t)(first * bs + within), (uint32_t)xfer_row, (uint32_t)rows,
                                          (uint32_t)(block_base + (b - b_first))});
                xfer_row += rows;
                b = e;
            }
            block_base += b_end - b_first;
        }

        // Then the descriptors: every run is split evenly into pieces of at most `piece` rows.
        // The tiled kernels launch the same number of tiles for every descriptor (that of the
        // largest), so a few descriptors that are larger than the rest leave most workgroups of a
        // launch without work -- 64 KiB blocks of which one pair in 70,000 happened to be adjacent
        // and was merged ran at 4.4 instead of 6.6 TB/s.  `piece` is therefore chosen among
        // block_tokens * 2^j (j of either sign) and the unit_bytes limit: the largest of them that
        // launches no more than 2 % above the fewest tiles.
        const uint64_t tile_bytes = (uint64_t)plan->tuning.block_threads * 16u;
        auto pieces_of = [](uint64_t rows, uint64_t piece) { return (rows + piece - 1) / piece; };
        uint64_t piece = max_rows, total_pieces = 0;
        {
            // run lengths with their counts (a table for the common short ones)
            constexpr uint32_t kTable = 4096;
            std::vector<uint32_t> table(kTable, 0);
            std::vector<std::pair<uint64_t, uint64_t>> lengths;      // (rows, how many runs)
            for (const kvl_unit_t &run : runs) {
                if (run.n_rows < kTable) ++table[run.n_rows];
                else lengths.emplace_back(run.n_rows, 1);
            }
            for (uint32_t n = 1; n < kTable; ++n)
                if (table[n]) lengths.emplace_back(n, table[n]);
            std::vector<uint64_t> candidates{max_rows};
            for (uint64_t c = bs; c < max_rows; c *= 2) candidates.push_back(c);
            for (uint64_t c = bs / 2; c >= 1 && c * max_row >= tile_bytes; c /= 2)      // blocks beyond the limit: halves, quarters, ...
                if (c < max_rows) candidates.push_back(c);
            std::vector<uint64_t> cost(candidates.size()), count(candidates.size());
            uint64_t least = UINT64_MAX;
            for (size_t j = 0; j < candidates.size(); ++j) {
                const uint64_t c = candidates[j];
                uint64_t n_pieces = 0, largest = 0;
                for (const auto &len : lengths) {
                    const uint64_t k = pieces_of(len.first, c);
                    n_pieces += k * len.second;
                    largest = std::max<uint64_t>(largest, (len.first + k - 1) / k);
                }
                count[j] = n_pieces;
                cost[j] = n_pieces * ((largest * max_row + tile_bytes - 1) / tile_bytes);
                least = std::min(least, cost[j]);
            }
            // the largest size within 2 % of the fewest tiles: a few tiles saved on ragged ends are
            // not worth many more descriptors
            uint64_t chosen = 0;
            for (size_t j = 0; j < candidates.size(); ++j) {
                if (cost[j] <= least + least / 50 && candidates[j] > chosen) {
                    chosen = candidates[j];
                    total_pieces = count[j];
                }
            }
            piece = chosen;
        }
        uint32_t longest = 0;
        if (total_pieces == runs.size()) {
            // nothing to split (the common case): the runs are the descriptors
            for (const kvl_unit_t &run : runs) longest = std::max(longest, run.n_rows);
            plan->units = std::move(runs);
        } else {
            plan->units.reserve((size_t)std::min<uint64_t>(total_pieces, (uint64_t)INT32_MAX));
            for (const kvl_unit_t &run : runs) {
                const uint64_t pieces = pieces_of(run.n_rows, piece);
                const uint64_t base = run.n_rows / pieces, extra = run.n_rows % pieces;
                const uint64_t within = run.pool_row % bs;
                uint64_t done = 0;
                for (uint64_t k = 0; k < pieces; ++k) {
                    const uint64_t n = base + (k < extra ? 1 : 0);
                    plan->units.push_back(kvl_unit_t{(uint32_t)(run.pool_row + done), (uint32_t)(run.xfer_row + done),
                                                     (uint32_t)n, (uint32_t)(run.block_index + (within + done) / bs)});
                    longest = std::max<uint32_t>(longest, (uint32_t)n);
                    done += n;
                }
            }
        }
        plan->blocks_touched = block_base;
        if (plan->units.size() > (size_t)INT32_MAX) { delete plan; return KVL_ERANGE; }
        plan->max_unit_rows = longest;
    } catch (const std::bad_alloc &) {
        delete plan;
        return KVL_ENOMEM;
    }

    uint64_t base = 0;
    for (uint32_t p = 0; p < layout->n_planes; ++p) {
        plan->plane_base[p] = base;
        base += plan->hit_tokens * layout->row_bytes[p];
    }
    plan->payload_bytes = base;

    if (!(flags & KVL_HOST_ONLY)) {
        rc = upload_units(plan);
        if (rc != KVL_OK) {
            kvl_plan_destroy(plan);
            return rc;
        }
    }
    *out = plan;
    return KVL_OK;
}

}  // namespace kvl

extern "C" {

int kvl_plan(const kvl_layout_t *layout, const kvl_request_t *requests, uint32_t n_req,
             uint32_t flags, kvl_plan_t **out) {
    return kvl::build(layout, requests, n_req, flags, nullptr, out);
}

int kvl_plan_tuned(const kvl_layout_t *layout, const kvl_request_t *requests, uint32_t n_req,
                   uint32_t flags, const kvl_tuning_t *tuning, kvl_plan_t **out) {
    return kvl::build(layout, requests, n_req, flags, tuning, out);
}

void kvl_plan_destroy(kvl_plan_t *plan) {
    if (!plan) return;
    if (plan->d_units) kvl::descriptor_release(plan);
    kvl::drop_stream_events(plan);          // of a plan that never owned a descriptor array
    for (hipStream_t s : plan->lanes) {
        // the lanes' work on this plan has normally ended (the stream the caller waits on follows
        // them); one that is still busy is waited for, it alone, since the plan's events go below
        if (hipStreamQuery(s) != hipSuccess) {
            (void)hipGetLastError();
            (void)hipStreamSynchronize(s);
        }
        if (plan->lane_cu_mask.empty()) kvl::return_lane(s, plan->device);
        else (void)hipStreamDestroy(s);
    }
    for (hipEvent_t e : plan->ev_lane_done) (void)hipEventDestroy(e);
    if (plan->ev_entry) (void)hipEventDestroy(plan->ev_entry);
    if (plan->ev_entry2) (void)hipEventDestroy(plan->ev_entry2);
    delete plan;
}

int kvl_plan_pair(const kvl_plan_t *g, const kvl_plan_t *s, kvl_plan_t **out) {
    if (!g || !s || !out) return KVL_EINVAL;
    *out = nullptr;
    if (!(g->flags & KVL_GATHER) || !(s->flags & KVL_SCATTER) || g->paired || s->paired) return KVL_EINVAL;
    const kvl_layout_t &a = g->layout, &b = s->layout;
    if (a.block_tokens != b.block_tokens || a.n_planes != b.n_planes || g->hit_tokens != s->hit_tokens)
        return KVL_EINVAL;
    for (uint32_t p = 0; p < a.n_planes; ++p)
        if (a.row_bytes[p] != b.row_bytes[p]) return KVL_EINVAL;
    kvl_plan_t *plan = new (std::nothrow) kvl_plan_t;
    if (!plan) return KVL_ENOMEM;
    plan->layout = a;
    plan->dst_pool_blocks = b.pool_blocks;
    plan->flags = KVL_GATHER | ((g->flags | s->flags) & KVL_HOST_ONLY) | (g->flags & s->flags & KVL_CALLER_SYNCS);
    plan->paired = true;
    plan->n_req = g->n_req;
    plan->hit_tokens = g->hit_tokens;
    plan->payload_bytes = g->payload_bytes;
    plan->vec16 = g->vec16;
    plan->tuning = g->tuning;
    plan->threads_chosen = g->threads_chosen;
    try {
        // both descriptor lists tile the token rows [0, T) in order: walk them together
        size_t i = 0, j = 0;
        uint64_t x = 0;
        uint32_t longest = 0;
        while (i < g->units.size() && j < s->units.size()) {
            const kvl_unit_t &u = g->units[i], &v = s->units[j];
            const uint64_t u_end = (uint64_t)u.xfer_row + u.n_rows, v_end = (uint64_t)v.xfer_row + v.n_rows;
            const uint64_t end = std::min(u_end, v_end);
            kvl_unit_t d{(uint32_t)(u.pool_row + (x - u.xfer_row)), (uint32_t)(v.pool_row + (x - v.xfer_row)),
                         (uint32_t)(end - x), 0};
            plan->units.push_back(d);
            longest = std::max(longest, d.n_rows);
            x = end;
            if (end == u_end) ++i;
            if (end == v_end) ++j;
        }
        plan->max_unit_rows = longest;
        // Both sides of a move are scattered over their pools; walking the descriptors in the
        // order of the destination rows makes the writes, the weaker side of the memory, run
        // forward through the pool (cfg3 and cfg4: 5.5-5.6 -> 6.1-6.2 TB/s of traffic).
        std::sort(plan->units.begin(), plan->units.end(),
                  [](const kvl_unit_t &a, const kvl_unit_t &b) { return a.xfer_row < b.xfer_row; });
    } catch (const std::bad_alloc &) {
        delete plan;
        return KVL_ENOMEM;
    }
    if (!(plan->flags & KVL_HOST_ONLY)) {
        int rc = kvl::upload_units(plan);
        if (rc != KVL_OK) {
            kvl_plan_destroy(plan);
            return rc;
        }
    }
    *out = plan;
    return KVL_OK;
}

int kvl_plan_set_tuning(kvl_plan_t *plan, const kvl_tuning_t *tuning) {
    if (!plan || !tuning) return KVL_EINVAL;
    kvl_tuning_t t = plan->tuning;
    if (tuning->block_threads) {
        if (!kvl::valid_block_threads(tuning->block_threads)) return KVL_EINVAL;
        t.block_threads = tuning->block_threads;
        plan->threads_chosen = true;
    }
    if (tuning->variant > kvl::kNumVariants) return KVL_EINVAL;
    t.variant = tuning->variant;
    t.max_groups = tuning->max_groups;
    plan->tuning = t;
    return KVL_OK;
}

int kvl_plan_payload_bytes(const kvl_plan_t *plan, uint64_t *bytes) {
    if (!plan || !bytes) return KVL_EINVAL;
    *bytes = plan->payload_bytes;
    return KVL_OK;
}

int kvl_plan_hit_tokens(const kvl_plan_t *plan, uint64_t *tokens) {
    if (!plan || !tokens) return KVL_EINVAL;
    *tokens = plan->hit_tokens;
    return KVL_OK;
}

int kvl_plan_fullblock_geometry(const kvl_plan_t *plan, uint64_t *full_block_bytes, uint64_t *n_full_blocks) {
    if (!plan || !full_block_bytes || !n_full_blocks) return KVL_EINVAL;
    uint64_t lb = 0;
    for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
        lb += (uint64_t)plan->layout.block_tokens * plan->layout.row_bytes[p];
    *full_block_bytes = lb * plan->layout.n_layers;
    *n_full_blocks = plan->blocks_touched;
    return KVL_OK;
}

int kvl_plan_n_units(const kvl_plan_t *plan, uint64_t *n) {
    if (!plan || !n) return KVL_EINVAL;
    *n = plan->units.size();
    return KVL_OK;
}

int kvl_plan_get_units(const kvl_plan_t *plan, kvl_unit_t *out, uint64_t capacity, uint64_t *n) {
    if (!plan || !n || (capacity && !out)) return KVL_EINVAL;
    *n = plan->units.size();
    const size_t k = (size_t)std::min<uint64_t>(capacity, plan->units.size());
    if (k) std::memcpy(out, plan->units.data(), k * sizeof(kvl_unit_t));
    return KVL_OK;
}

int kvl_plan_get_chunks(const kvl_plan_t *plan, uint64_t chunk_bytes, kvl_chunk_t *out,
                        uint64_t capacity, uint64_t *n) {
    if (!plan || !n || (capacity && !out)) return KVL_EINVAL;
    std::vector<kvl_chunk_t> c;
    int rc;
    try {
        rc = kvl::make_chunks(plan, chunk_bytes, c);
    } catch (const std::bad_alloc &) {
        return KVL_ENOMEM;
    }
    if (rc != KVL_OK) return rc;
    *n = c.size();
    const size_t k = (size_t)std::min<uint64_t>(capacity, c.size());
    if (k) std::memcpy(out, c.data(), k * sizeof(kvl_chunk_t));
    return KVL_OK;
}

int kvl_check_buffer(const void *ptr, uint64_t bytes, int allow_host) {
    if (!ptr) return bytes ? KVL_EINVAL : KVL_OK;
    hipPointerAttribute_t a{};
    if (hipPointerGetAttributes(&a, ptr) != hipSuccess) {
        (void)hipGetLastError();                     // not an error of ours: the pointer is unknown to HIP
        return KVL_EINVAL;
    }
    const bool on_device = a.type == hipMemoryTypeDevice || a.type == hipMemoryTypeManaged;
    if (!on_device && a.type != hipMemoryTypeHost) return KVL_EINVAL;   // unregistered (pageable) host memory, arrays
    if (a.type == hipMemoryTypeHost && !(allow_host && a.devicePointer)) return KVL_EINVAL;
    // the extent of the allocation, where the runtime knows it (it does for its own device and
    // pinned host allocations)
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void *>(ptr)) != hipSuccess) {
        (void)hipGetLastError();
        return KVL_OK;                               // extent unknown: nothing more to check
    }
    const uintptr_t p = reinterpret_cast<uintptr_t>(ptr), b = reinterpret_cast<uintptr_t>(base);
    return (p >= b && bytes <= size && p - b <= size - bytes) ? KVL_OK : KVL_ESPACE;
}

void kvl_release_cached_memory(void) {
    std::vector<kvl::CachedBuffer> drop;
    std::vector<kvl::PooledLane> lanes;
    std::vector<std::pair<hipEvent_t, int>> events;
    {
        std::lock_guard<std::mutex> lock(kvl::g_cache_mutex);
        kvl::reap_retired(true);                    // waits for the kernels of destroyed plans, nothing else
        drop.swap(kvl::g_cache);
        lanes.swap(kvl::g_lanes);
        events.swap(kvl::g_events);
    }
    for (const kvl::CachedBuffer &b : drop) (void)hipFree(b.ptr);
    for (const kvl::PooledLane &l : lanes) {
        (void)hipStreamSynchronize(l.stream);
        (void)hipStreamDestroy(l.stream);
    }
    for (const auto &e : events) (void)hipEventDestroy(e.first);
    // the upload streams and their pinned staging buffers come back on the next plan
    std::lock_guard<std::mutex> lock(kvl::g_upload_mutex);
    for (kvl::Uploader &u : kvl::g_uploaders) {
        if (u.bounce) (void)hipHostFree(u.bounce);
        if (u.stream) (void)hipStreamDestroy(u.stream);
        u = kvl::Uploader{};
    }
}

const char *kvl_strerror(int code) {
    switch (code) {
        case KVL_OK: return "ok";
        case KVL_EINVAL: return "invalid argument";
        case KVL_ERANGE: return "block id, table length or size out of range";
        case KVL_EALIAS: return "destination block named twice in a scatter plan";
        case KVL_ESPACE: return "buffer, staging area or chunk too small";
        case KVL_EHIP: return "HIP call failed";
        case KVL_ENOMEM: return "out of host memory";
        case KVL_ENOSYS: return "not available in the HIP runtime of this process";
        default: return "unknown kvl error";
    }
}

int kvl_last_hip_error(void) { return (int)kvl::g_last_hip; }

const char *kvl_last_hip_error_string(void) { return hipGetErrorString(kvl::g_last_hip); }

const char *kvl_version(void) { return "kvl 0.1 (gfx950)"; }

}  // extern "C"
