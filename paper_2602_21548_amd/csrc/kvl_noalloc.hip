// kvl_unpack_layer_noalloc: the scatter of one layer for callers that may not allocate.
//
// kvl_plan + kvl_unpack_layer keep a batch's copy descriptors in a device buffer the library
// allocates per plan.  This variant takes the batch itself instead of a plan and keeps the
// descriptors in a fixed array in device memory that is part of the library's code object, so
// the call touches no allocator: no hipMalloc, no hipFree, no stream or event creation after the
// first call on a device.  The copy kernels are the ones kvl_unpack_layer launches; they read the
// descriptors through the pointer they are given, as they do there.
#include <cstring>
#include <mutex>

#include "kvl_internal.h"

namespace kvl {
namespace {

constexpr uint32_t kMaxUnits = KVL_NOALLOC_MAX_UNITS;
constexpr int kMaxDevices = 64;

// One copy of this array lives on every GPU the library's code object is loaded on, at an
// address of its own; it keeps the last call's descriptors until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress: kernels get the address that call
// returned, never the name.
static __device__ __align__(256) kvl_unit_t scratch[kMaxUnits];

// Host-side staging for the upload.  Reused by every call on every device, so a call first waits
// for the previous upload out of it (g_bounce_busy: the event that follows that upload, on whichever
// device it ran) to finish.
static kvl_unit_t g_bounce[kMaxUnits];
static hipEvent_t g_bounce_busy = nullptr;

struct DeviceState {
    kvl_unit_t *units = nullptr;       // device address of `scratch` on this GPU
    hipEvent_t uploaded = nullptr;     // the last upload out of g_bounce has finished
    hipEvent_t kernels_done = nullptr; // the last call's kernels have finished reading `units`
};
DeviceState g_dev[kMaxDevices];
std::mutex g_mutex;                    // serialises the calls of a process (they share g_bounce and `scratch`)

// First call on a device, with that device current.
int setup(int device, DeviceState **out) {
    DeviceState &d = g_dev[device];
    if (!d.units) {
        kvl_unit_t *ptr = nullptr;
        KVL_HIP(hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch)));
        if (!ptr) return KVL_EHIP;
        hipEvent_t a = nullptr, b = nullptr;
        KVL_HIP(hipEventCreateWithFlags(&a, hipEventDisableTiming));
        hipError_t e = hipEventCreateWithFlags(&b, hipEventDisableTiming);
        if (e != hipSuccess) {
            (void)hipEventDestroy(a);
            set_hip_error(e);
            return KVL_EHIP;
        }
        d.uploaded = a;
        d.kernels_done = b;
        d.units = ptr;
    }
    *out = &d;
    return KVL_OK;
}

}  // namespace
}  // namespace kvl

extern "C" {

int kvl_unpack_layer_noalloc(const kvl_layout_t *layout, const kvl_request_t *requests, uint32_t n_req,
                             uint32_t flags, const void *xfer, uint64_t xfer_bytes,
                             void *const *pool_planes, void *stream) {
    using namespace kvl;
    if (!layout || !pool_planes || (n_req && !requests)) return KVL_EINVAL;
    if (flags & ~(KVL_NO_MERGE | KVL_TOKENS_APPEND | KVL_TOKENS_ALL | KVL_NO_POINTER_CHECKS)) return KVL_EINVAL;
    // descriptors on the host: validation, layout and run merging are those of kvl_plan
    kvl_plan_t *plan = nullptr;
    // (KVL_CALLER_SYNCS: the kernels are followed by this file's own event, not by the plan's)
    int rc = kvl_plan(layout, requests, n_req, flags | KVL_SCATTER | KVL_HOST_ONLY | KVL_CALLER_SYNCS, &plan);
    if (rc != KVL_OK) return rc;
    const size_t n_units = plan->units.size();
    if (n_units > kMaxUnits) rc = KVL_ESPACE;                    // the fixed array cannot hold this batch
    else if (xfer_bytes < plan->payload_bytes) rc = KVL_ESPACE;
    else if (n_units && !xfer) rc = KVL_EINVAL;
    if (rc != KVL_OK || n_units == 0) {
        kvl_plan_destroy(plan);
        return rc;
    }
    hipStream_t s = (hipStream_t)stream;
    int device = -1;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess || device < 0 || device >= kMaxDevices) {
        if (e != hipSuccess) set_hip_error(e);
        kvl_plan_destroy(plan);
        return e != hipSuccess ? KVL_EHIP : KVL_EINVAL;
    }
    plan->device = device;
    rc = check_pool(plan, pool_planes, plan->layout.pool_blocks);
    if (rc == KVL_OK) rc = check_buffer(plan, xfer, plan->payload_bytes, true);
    if (rc == KVL_OK) {
        std::lock_guard<std::mutex> lock(g_mutex);
        DeviceState *d = nullptr;
        rc = setup(device, &d);
        auto hip = [&rc](hipError_t err) {
            if (err != hipSuccess && rc == KVL_OK) {
                set_hip_error(err);
                rc = KVL_EHIP;
            }
            return err == hipSuccess;
        };
        if (rc == KVL_OK) {
            const size_t bytes = n_units * sizeof(kvl_unit_t);
            // the staging array is free once the previous upload has left it, the device array once
            // the previous call's kernels (on whatever stream they ran) have finished
            // (an event that was never recorded counts as finished)
            bool ok = !g_bounce_busy || hip(hipEventSynchronize(g_bounce_busy));
            if (ok) {
                std::memcpy(g_bounce, plan->units.data(), bytes);
                ok = hip(hipStreamWaitEvent(s, d->kernels_done, 0)) &&
                     hip(hipMemcpyAsync(d->units, g_bounce, bytes, hipMemcpyHostToDevice, s));
                if (ok) {
                    g_bounce_busy = d->uploaded;
                    ok = hip(hipEventRecord(d->uploaded, s));
                    if (!ok) (void)hipStreamSynchronize(s);      // nothing follows the upload: wait for it here
                }
            }
            if (ok) {
                plan->d_units = d->units;            // borrowed: taken back before the plan is destroyed
                uintptr_t xp[KVL_MAX_PLANES];
                for (uint32_t p = 0; p < plan->layout.n_planes; ++p)
                    xp[p] = reinterpret_cast<uintptr_t>(xfer) + plan->plane_base[p];
                int lrc = launch_units(plan, false, 0, (uint32_t)n_units, 0, plan->layout.n_planes, pool_planes, xp, s,
                                       is_host_memory(plan, xfer));
                plan->d_units = nullptr;
                if (rc == KVL_OK) rc = lrc;
                // recorded even after a failed launch: the upload above is in flight on s
                hip(hipEventRecord(d->kernels_done, s));
            }
        }
    }
    kvl_plan_destroy(plan);
    return rc;
}

}  // extern "C"
