// Device side: the pack/unpack kernels and their launcher.
#pragma once

#include <hip/hip_runtime_api.h>

#include "plan.hpp"

namespace tp {

// Enqueues one planned launch on `stream`.  Returns hipSuccess or the launch error.
hipError_t enqueue(const Launch& launch, bool unpack, hipStream_t stream);

// Enqueues one batched launch (see plan.hpp: BatchParams).
hipError_t enqueue_batch(const BatchParams& batch, bool unpack, hipStream_t stream);

}  // namespace tp
