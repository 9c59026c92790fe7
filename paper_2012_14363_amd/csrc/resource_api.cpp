// C ABI of the resource cache (see include/tp_pack.h) and its HIP backend.  Paper Sec. 5.
#include "tp_pack.h"

#include <hip/hip_runtime_api.h>

#include "resource_cache.hpp"
#include "status.hpp"

namespace tp {

namespace {

// Creates on the current device, which acquire() has just read `device` from.
bool hip_create(int kind, int /*device*/, size_t bytes, void** handle, void** gpu_view) {
    hipError_t e = hipErrorInvalidValue;
    *gpu_view = nullptr;
    switch (kind) {
    case kResDevice:
        e = hipMalloc(handle, bytes);
        *gpu_view = *handle;
        break;
    case kResPinned:
        // mapped into the device's address space so kernels can read and write it directly
        e = hipHostMalloc(handle, bytes, hipHostMallocMapped);
        if (e == hipSuccess) {
            e = hipHostGetDevicePointer(gpu_view, *handle, 0);
            if (e != hipSuccess) (void)hipHostFree(*handle);
        }
        break;
    case kResStream: {
        hipStream_t s = nullptr;
        e = hipStreamCreateWithFlags(&s, hipStreamNonBlocking);  // default priority
        *handle = s;
        break;
    }
    case kResEvent: {
        hipEvent_t ev = nullptr;
        e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
        *handle = ev;
        break;
    }
    default:
        return false;
    }
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *handle = nullptr;
        return false;
    }
    return true;
}

void hip_destroy(int kind, int device, void* handle) {
    int before = -1;
    const bool switched = hipGetDevice(&before) == hipSuccess && before != device && hipSetDevice(device) == hipSuccess;
    switch (kind) {
    case kResDevice: (void)hipFree(handle); break;
    case kResPinned: (void)hipHostFree(handle); break;
    case kResStream: (void)hipStreamDestroy(static_cast<hipStream_t>(handle)); break;
    case kResEvent: (void)hipEventDestroy(static_cast<hipEvent_t>(handle)); break;
    default: break;
    }
    if (switched) (void)hipSetDevice(before);
}

int hip_current_device() {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return device;
}

}  // namespace

ResourceCache& library_resources() {
    static ResourceCache* cache = new ResourceCache(ResourceBackend{hip_create, hip_destroy, hip_current_device});
    return *cache;
}

}  // namespace tp

extern "C" {

int tp_resource_acquire(int kind, int64_t bytes, void** handle) {
    return tp::library_resources().acquire(kind, bytes, handle);
}

int tp_resource_release(int kind, void* handle) { return tp::library_resources().release(kind, handle); }

int tp_resource_trim(int64_t* bytes_freed) {
    const int64_t bytes = tp::library_resources().trim();
    if (bytes_freed) *bytes_freed = bytes;
    return tp::kSuccess;
}

int tp_resource_stats(int kind, tp_resource_counts* out) {
    if (!out || kind < 0 || kind >= tp::kResKinds) return tp::kErrArg;
    const tp::ResourceCounts c = tp::library_resources().counts(kind);
    out->hits = c.hits;
    out->misses = c.misses;
    out->idle = c.idle;
    out->leased = c.leased;
    out->idle_bytes = c.idle_bytes;
    out->leased_bytes = c.leased_bytes;
    return tp::kSuccess;
}

}  // extern "C"
