// Pack/unpack entry points for callers inside the library that bring device memory of their own
// (memory the runtime's pointer queries need not know, such as a device-side global array).
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstdint>

#include "tp_pack.h"

namespace tp {

// tp_pack_async / tp_unpack_async whose contiguous buffer is [device_buf, device_buf + size) of
// device memory the caller vouches for: it is not queried, everything else is checked as usual.
int transfer_with_device_buffer(bool unpack, const void* typed_buf, int64_t count, tp_type t, void* device_buf,
                                int64_t size, int64_t* position, hipStream_t stream);

// Enqueues one dense copy of `bytes` from device memory the caller vouches for to
// packed_buf + position (device or mapped host memory, checked as for tp_pack).  Same kernels as a
// fully dense datatype; neither allocates nor synchronizes.
int copy_device_buffer_to_packed(const void* device_src, int64_t bytes, void* packed_buf, int64_t packed_size,
                                 int64_t position, hipStream_t stream);

}  // namespace tp
