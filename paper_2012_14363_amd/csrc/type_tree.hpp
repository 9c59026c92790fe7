// Datatype tree: one immutable node per constructor call (paper Sec. 2), with the
// size and bounds every later stage needs computed once at construction.
#pragma once

#include <atomic>
#include <cstdint>
#include <memory>
#include <mutex>
#include <vector>

#include "strided_block.hpp"

namespace tp {

enum class Kind : uint8_t { Named, Contiguous, Vector, Hvector, Subarray };

struct TypeNode {
    Kind kind = Kind::Named;
    int64_t count = 0;        // contiguous / vector / hvector
    int64_t blocklength = 0;  // vector / hvector
    int64_t stride = 0;       // vector: in elements of old; hvector: in bytes
    int order = 0;            // subarray: 0 = C, 1 = Fortran
    std::vector<int64_t> sizes, subsizes, starts;
    std::shared_ptr<const TypeNode> old;

    int64_t size = 0;  // data bytes of one object
    int64_t lb = 0;    // lower bound, bytes from the origin
    int64_t ub = 0;    // upper bound
    int64_t extent() const { return ub - lb; }

    // Filled by commit (Sec. 3: the result is cached with the datatype).  `committed` is set
    // last, with release order, so a thread that sees it also sees `block`.
    mutable std::once_flag commit_once;
    mutable std::atomic<bool> committed{false};
    mutable int commit_status = 0;
    mutable StridedBlock block;
};

using TypePtr = std::shared_ptr<const TypeNode>;

// Constructors.  Return a TP_* status; on success *out holds the node.
int make_named(int64_t size_bytes, TypePtr* out);
int make_contiguous(int64_t count, const TypePtr& old, TypePtr* out);
int make_vector(int64_t count, int64_t blocklength, int64_t stride, bool stride_in_bytes, const TypePtr& old,
                TypePtr* out);
int make_subarray(int ndims, const int* sizes, const int* subsizes, const int* starts, int order, const TypePtr& old,
                  TypePtr* out);

// Handle table: int32 handles -> nodes.  Slots are recycled; a generation count in
// the upper bits makes a stale handle invalid rather than an alias of a newer type.
class HandleTable {
public:
    HandleTable();
    int32_t insert(TypePtr node);
    TypePtr lookup(int32_t handle) const;  // nullptr when invalid
    bool erase(int32_t handle);            // false when invalid or predefined
    static HandleTable& instance();

private:
    static constexpr int kIndexBits = 20;
    struct Slot {
        TypePtr node;
        uint32_t generation = 0;
    };
    mutable std::mutex mu_;
    std::vector<Slot> slots_;
    std::vector<uint32_t> free_;
};

}  // namespace tp
