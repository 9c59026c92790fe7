// Commit-time pipeline of paper Sec. 3: translation of a datatype tree into the
// Type IR (Sec. 3.1), canonicalization (Sec. 3.2) and conversion into a
// StridedBlock (Sec. 3.3, Alg. 5).
#pragma once

#include <cstdint>
#include <vector>

#include "strided_block.hpp"
#include "type_tree.hpp"

namespace tp {

// One level of the Type IR.  Sec. 3.1 has two kinds of TypeData:
//   DenseData  {offset, extent}        - `extent` contiguous bytes, no child
//   StreamData {offset, stride, count} - `count` copies of the single child, `stride` bytes apart
// Because every level has at most one child the hierarchy is a chain, kept here
// as a vector from the root (index 0) down to the DenseData leaf (last).
struct Level {
    bool dense = false;
    int64_t offset = 0;
    int64_t stride = 0;  // StreamData only
    int64_t count = 0;   // StreamData only
    int64_t extent = 0;  // DenseData only
};
using Chain = std::vector<Level>;

// Sec. 3.1 translation rules (from_named / from_contiguous / from_vector /
// from_hvector / from_subarray).
Chain translate(const TypeNode& type);

// The three order-preserving passes of Sec. 3.2; each returns true if it changed the chain.
bool dense_folding(Chain& chain);   // Alg. 2
bool stream_elision(Chain& chain);  // Alg. 3, applied to every count-1 stream
bool stream_flatten(Chain& chain);  // Alg. 4
void simplify(Chain& chain);        // Alg. 1 without the sort step

// Alg. 5.  Returns a TP_* status (kErrRange if the chain has more than kMaxDims levels).
int strided_block(const Chain& chain, StridedBlock* out);

// translate + simplify + strided_block; an empty type gives ndims 1, counts[0] 0.
int canonicalize(const TypeNode& type, StridedBlock* out);

// Commit: the three phases above, run once per node whichever threads ask, and cached in it
// (Sec. 3: the result is kept with the datatype).  Returns the node's commit status.
int commit(const TypeNode& node);

}  // namespace tp
