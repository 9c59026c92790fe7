// What one pack/unpack call has learned about the memory its pointers lie in.
//
// Each call checks that the first, the lowest and the highest byte it would touch on either side
// are GPU-addressable.  Asking the runtime for every such byte would cost a batched call several
// queries per request; instead the first query about an address also fetches the bounds of the
// allocation that holds it, and later addresses inside a known allocation need no query at all.
// Header-only and free of HIP: the query is a function pointer, so tests can supply a fake one.
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "status.hpp"

namespace tp {

struct MemRange {
    uintptr_t lo = 0, hi = 0;  // [lo, hi): the allocation, or as much of it as is known
    bool host = false;         // pinned host memory mapped for the GPU (else device memory)
    ptrdiff_t view_delta = 0;  // address kernels use = address + view_delta
};

class BufferMap {
public:
    // Fills *range with the allocation that holds `p` (it must contain p).  Returns kSuccess,
    // kErrBuffer if the GPU cannot address p, or kErrOther on a runtime failure.
    using Query = int (*)(const void* p, MemRange* range);

    // `query` null: every address is taken as device memory, unchecked.
    explicit BufferMap(Query query) : query_(query) {}

    // Resolves `p` to the address kernels use for it.  `allow_host`: mapped host memory is
    // acceptable (the contiguous side of a call only); *is_host (may be null) tells which it is.
    int locate(const void* p, bool allow_host, const char** view, bool* is_host = nullptr) {
        if (is_host) *is_host = false;
        if (!query_) {
            *view = static_cast<const char*>(p);
            return kSuccess;
        }
        const uintptr_t a = reinterpret_cast<uintptr_t>(p);
        const MemRange* r = find(a);
        if (!r) {
            MemRange fresh;
            const int rc = query_(p, &fresh);
            if (rc != kSuccess) return rc;
            if (!(fresh.lo <= a && a < fresh.hi)) {  // a query that answers about other memory: trust only p
                fresh.lo = a;
                fresh.hi = a + 1;
            }
            known_.push_back(fresh);
            r = &known_.back();
        }
        if (r->host && !allow_host) return kErrBuffer;
        if (is_host) *is_host = r->host;
        *view = static_cast<const char*>(p) + r->view_delta;
        return kSuccess;
    }

    // Checks that `p` is addressable, without needing its view.
    int check(const void* p, bool allow_host) {
        const char* ignored = nullptr;
        return locate(p, allow_host, &ignored);
    }

    // Memory the library itself vouches for (its own buffers): addresses inside need no query.
    void add_known(const MemRange& range) { known_.push_back(range); }

    size_t known_ranges() const { return known_.size(); }

private:
    const MemRange* find(uintptr_t a) const {
        for (const MemRange& r : known_)
            if (r.lo <= a && a < r.hi) return &r;
        return nullptr;
    }
    Query query_;
    std::vector<MemRange> known_;
};

}  // namespace tp
