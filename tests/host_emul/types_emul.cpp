// The library's datatype tree, handle table, canonicalizer and commit compiled for the host, for
// tests only: a threaded exercise of what the C ABI does with them, so that a build with a
// sanitizer (thread or address) sees these paths with the host compiler.
#include <atomic>
#include <cstdint>
#include <thread>
#include <vector>

#include "canon.hpp"
#include "status.hpp"
#include "type_tree.hpp"

extern "C" {

// `threads` threads, `rounds` times each: build vector-of-contiguous types through the handle
// table, commit one node from every thread at once, look handles up while others free theirs, and
// check every canonical form against the closed form of that construction.  Returns the mismatches.
int64_t types_emul_hammer(int threads, int rounds) {
    using namespace tp;
    std::atomic<int64_t> bad{0};
    HandleTable& table = HandleTable::instance();
    // one node shared by all threads: its commit must run once and be seen whole by everyone
    TypePtr byte = table.lookup(0), shared;
    if (!byte || make_vector(64, 8, 512, false, byte, &shared) != kSuccess) return -1;
    const int32_t shared_handle = table.insert(shared);
    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t) {
        pool.emplace_back([&, t] {
            for (int r = 0; r < rounds; ++r) {
                const int64_t run = 1 + (t + r) % 7, rows = 2 + r % 5;
                TypePtr inner, outer;
                if (make_contiguous(run, byte, &inner) != kSuccess ||
                    make_vector(rows, 1, 100, true, inner, &outer) != kSuccess) {
                    ++bad;
                    continue;
                }
                const int32_t hi = table.insert(inner), ho = table.insert(outer);
                if (hi < 12 || ho < 12 || hi == ho) ++bad;
                if (!table.erase(hi)) ++bad;                 // the derived type keeps its own reference
                if (table.lookup(hi)) ++bad;                 // a stale handle stays invalid
                const TypePtr got = table.lookup(ho);
                if (!got || commit(*got) != kSuccess || !got->committed.load(std::memory_order_acquire)) {
                    ++bad;
                } else {
                    const StridedBlock& b = got->block;
                    if (b.ndims != 2 || b.counts[0] != run || b.counts[1] != rows || b.strides[1] != 100 || b.start != 0) ++bad;
                }
                const TypePtr sh = table.lookup(shared_handle);
                if (!sh || commit(*sh) != kSuccess) ++bad;
                else if (sh->block.ndims != 2 || sh->block.counts[0] != 8 || sh->block.counts[1] != 64 || sh->block.strides[1] != 512) ++bad;
                if (!table.erase(ho) || table.erase(ho)) ++bad;   // the second erase must fail
            }
        });
    }
    for (std::thread& th : pool) th.join();
    if (!table.erase(shared_handle)) ++bad;
    return bad.load();
}

}  // extern "C"
