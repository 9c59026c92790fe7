// StridedBlock: the canonical form of a strided datatype (paper Sec. 3.3).
#pragma once

#include <cstdint>

namespace tp {

constexpr int kMaxDims = 16;

// counts[0] contiguous bytes (strides[0] == 1); dimension d+1 repeats dimension d
// counts[d+1] times, strides[d+1] bytes apart.  `start` is the displacement of the
// first byte from the type's origin.  Dimensions stay in nesting order, so a
// row-major walk over counts (last dimension slowest) visits bytes in MPI
// type-map order.  An empty type has ndims == 1 and counts[0] == 0.
struct StridedBlock {
    int ndims = 0;
    int64_t start = 0;
    int64_t counts[kMaxDims] = {};
    int64_t strides[kMaxDims] = {};
};

}  // namespace tp
