// Staged delivery of packed data to host memory through a staging buffer that is part of the
// library's device image instead of an allocation: the entry point for callers that must not
// allocate (see include/tp_pack.h: tp_pack_host_static).
#include "tp_pack.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "status.hpp"
#include "transfer.hpp"

namespace {

using namespace tp;

// The staging buffer.  Every GPU the library runs on holds its own copy of this array, at its own
// address, from the moment the library's code is loaded there until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[TP_STATIC_STAGING_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_address[kMaxDevices] = {};   // per device; filled on the first call on that device

// The array's address on the current device.
int scratch_on_current_device(void** address) {
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) {
        (void)hipGetLastError();
        return kErrOther;
    }
    std::lock_guard<std::mutex> hold(g_lock);
    if (!g_scratch_address[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return kErrOther;
        }
        g_scratch_address[device] = p;
    }
    *address = g_scratch_address[device];
    return kSuccess;
}

}  // namespace

extern "C" int tp_pack_host_static(const void* inbuf, int incount, tp_type t, void* host_outbuf, int64_t outsize,
                                   int64_t* position, void* hip_stream) {
    if (!position) return kErrArg;
    int64_t bytes = 0;
    int rc = tp_pack_size(incount, t, &bytes);
    if (rc != kSuccess) return rc;
    if (bytes > TP_STATIC_STAGING_BYTES) return kErrRange;
    if (*position < 0 || outsize < 0) return kErrArg;
    if (bytes > outsize - *position) return kErrTruncate;
    if (bytes > 0 && !host_outbuf) return kErrBuffer;
    void* staging = nullptr;
    if ((rc = scratch_on_current_device(&staging)) != kSuccess) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // gather into the staging array (always from its first byte: nothing of an earlier call is kept),
    // then one dense copy of exactly these bytes to the host buffer, both as kernels on the stream
    int64_t staged = 0;
    rc = transfer_with_device_buffer(false, inbuf, incount, t, staging, TP_STATIC_STAGING_BYTES, &staged, stream);
    if (rc != kSuccess) {
        // only a launch the runtime refused can fail after earlier launches of the call went out
        if (rc == kErrOther) (void)hipStreamSynchronize(stream);
        return rc;
    }
    rc = copy_device_buffer_to_packed(staging, bytes, host_outbuf, outsize, *position, stream);
    if (rc != kSuccess) {
        (void)hipStreamSynchronize(stream);   // the gather may be in flight: leave the array quiet
        return rc;
    }
    if (hipStreamSynchronize(stream) != hipSuccess) {
        (void)hipGetLastError();
        return kErrOther;
    }
    *position += bytes;
    return kSuccess;
}
