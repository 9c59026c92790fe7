// Host emulation of the planned kernel launches, for tests only.
//
// Compiles the library's planner (plan.cpp) and the very same per-thread kernel
// body (tile_body.hpp) with the host compiler and runs every workgroup and thread
// of every launch sequentially, with each memory access checked: inside the
// buffer it belongs to, and no destination byte written a second time with a
// different value (the last word of a run may overlap its neighbour, which writes
// the same bytes twice).  It exists so that index and bounds mistakes show up on
// the CPU instead of as a GPU memory fault.  Nothing in the product path uses it.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "plan.hpp"
#include "status.hpp"
#include "tile_body.hpp"

namespace {

struct Checks {
    const char* typed_lo;
    const char* typed_hi;
    const char* packed_lo;
    const char* packed_hi;
    uint8_t* write_count;  // one counter per destination byte, or null
    const char* dst_lo;
    int64_t oob = 0;        // accesses that leave their buffer
    int64_t unaligned = 0;  // accesses at an address that is no multiple of their width (legal)
    int64_t rewritten = 0;  // destination bytes written again with a different value
    int64_t duplicates = 0; // destination bytes written again with the same value
    int64_t loads = 0;      // all loads
    const char* prefetched_lo = nullptr;  // what the read-only passes of a staged unpack cover
    const char* prefetched_hi = nullptr;
    // staged unpack: the last read-only pass, and the tile a store pass is in; a packed byte read by
    // tile t of a store pass must lie in tile t of that read-only pass (same workgroup, same XCD's L2)
    tp::PrefetchParams pass{};
    bool in_store_pass = false;
    uint32_t tile = 0;
    int64_t misplaced = 0;
};

struct HostMem {
    Checks* c;
    bool inside(const char* p, size_t n) const {
        return (p >= c->typed_lo && p + n <= c->typed_hi) || (p >= c->packed_lo && p + n <= c->packed_hi);
    }
    template <class W>
    W load(const char* p) const {
        W v{};
        c->loads++;
        if (c->in_store_pass && p >= c->packed_lo && p < c->packed_hi) {
            const char* lo = c->pass.base + static_cast<uint64_t>(c->tile) * c->pass.tile_bytes;
            if (c->pass.base == nullptr || p < lo || p + sizeof(W) > lo + c->pass.tile_bytes) c->misplaced++;
        }
        if (!inside(p, sizeof(W))) { c->oob++; return v; }
        if (reinterpret_cast<uintptr_t>(p) % sizeof(W)) c->unaligned++;
        std::memcpy(&v, p, sizeof(W));
        return v;
    }
    template <class W>
    void store(char* p, const W& v) const {
        if (!inside(p, sizeof(W))) { c->oob++; return; }
        if (reinterpret_cast<uintptr_t>(p) % sizeof(W)) c->unaligned++;
        if (c->write_count) {
            const char* bytes = reinterpret_cast<const char*>(&v);
            for (size_t i = 0; i < sizeof(W); ++i)
                if (c->write_count[p - c->dst_lo + static_cast<long>(i)]++) {
                    if (p[i] != bytes[i]) c->rewritten++; else c->duplicates++;
                }
        }
        std::memcpy(p, &v, sizeof(W));
    }
    template <class W>
    void consume(const W&) const {}
};

// Visitor for dispatch_launch: run every workgroup and thread of the variant a launch names.
template <bool UNPACK>
struct RunLaunch {
    const tp::KParams* p;
    uint32_t nblocks;
    HostMem mem;
    template <int WLOG2, int UX, int UR, int NRD>
    void operator()() {
        for (uint32_t b = 0; b < nblocks; ++b) {
            mem.c->tile = b;
            for (uint32_t t = 0; t < static_cast<uint32_t>(tp::kBlockThreads); ++t)
                tp::tile_thread<WLOG2, UX, UR, UNPACK, NRD>(*p, b, t, mem);
        }
    }
};

// A transposing launch: per workgroup, every thread's first phase, then every thread's second
// phase (the barrier), with the workgroup's LDS tile as a host array.  Reports an LDS index
// outside the tile as an out-of-bounds access.
template <int WLOG2, bool UNPACK>
void run_xpose_words(const tp::Launch& l, HostMem mem) {
    using W = typename tp::WordOf<WLOG2>::type;
    using Tile = tp::XposeTile<WLOG2>;
    const tp::XParams& x = l.x;
    if (x.ew == 0 || x.te_a == 0 || x.te_b == 0 || x.fa_log2 > 8 || x.fb_log2 > 8 ||
        x.pitch < x.te_a * x.ew || uint64_t{x.te_b} * x.pitch > static_cast<uint64_t>(Tile::kLdsWords)) {
        mem.c->oob++;
        return;
    }
    std::vector<W> lds(static_cast<size_t>(Tile::kLdsWords));
    for (uint32_t b = 0; b < l.nblocks; ++b) {
        std::memset(lds.data(), 0x5C, lds.size() * sizeof(W));
        // the same choice of variant as the device launcher's
        const bool square = tp::xpose_is_square(l.x, WLOG2);
        for (uint32_t t = 0; t < static_cast<uint32_t>(tp::kBlockThreads); ++t) {
            if (square) tp::xpose_phase<WLOG2, UNPACK, true, true>(l.x, b, t, mem, lds.data());
            else tp::xpose_phase<WLOG2, UNPACK, true, false>(l.x, b, t, mem, lds.data());
        }
        for (uint32_t t = 0; t < static_cast<uint32_t>(tp::kBlockThreads); ++t) {
            if (square) tp::xpose_phase<WLOG2, UNPACK, false, true>(l.x, b, t, mem, lds.data());
            else tp::xpose_phase<WLOG2, UNPACK, false, false>(l.x, b, t, mem, lds.data());
        }
    }
}

bool run_xpose(const tp::Launch& l, bool unpack, HostMem mem) {
    switch (l.word_log2) {
    case 0: unpack ? run_xpose_words<0, true>(l, mem) : run_xpose_words<0, false>(l, mem); return true;
    case 1: unpack ? run_xpose_words<1, true>(l, mem) : run_xpose_words<1, false>(l, mem); return true;
    case 2: unpack ? run_xpose_words<2, true>(l, mem) : run_xpose_words<2, false>(l, mem); return true;
    case 3: unpack ? run_xpose_words<3, true>(l, mem) : run_xpose_words<3, false>(l, mem); return true;
    case 4: unpack ? run_xpose_words<4, true>(l, mem) : run_xpose_words<4, false>(l, mem); return true;
    default: return false;
    }
}

// Runs one planned launch of either kind; false if it names no kernel variant.
bool run_launch(const tp::Launch& l, bool unpack, Checks* c) {
    if (l.grid > l.nblocks) return false;
    if (l.kind == tp::kXpose) return run_xpose(l, unpack, HostMem{c});
    if (l.kind == tp::kPrefetch) {
        // the launcher's checks, then every tile (whichever workgroup takes it) and thread
        const tp::PrefetchParams& f = l.f;
        if (!unpack || !f.base || f.bytes < 16 || f.tile_bytes < 16 || (f.tile_bytes & (f.tile_bytes - 1)) || f.ntiles != l.nblocks ||
            (f.bytes + f.tile_bytes - 1) / f.tile_bytes != f.ntiles)
            return false;
        c->pass = f;
        c->in_store_pass = false;
        c->prefetched_lo = c->prefetched_lo ? std::min(c->prefetched_lo, f.base) : f.base;
        c->prefetched_hi = std::max(c->prefetched_hi, f.base + f.bytes);
        const uint32_t grid = l.grid ? l.grid : l.nblocks;
        const int64_t loads_before = c->loads;
        for (uint32_t b = 0; b < grid; ++b)
            for (uint32_t t = 0; t < static_cast<uint32_t>(tp::kBlockThreads); ++t)
                tp::prefetch_thread(f, b, grid, t, HostMem{c});
        // every 16-byte word of the bytes is loaded exactly once (the last may be pulled back)
        if (c->loads - loads_before != static_cast<int64_t>((f.bytes + 15) / 16)) c->oob++;
        return true;
    }
    const tp::KParams p = tp::kernel_params(l);
    // a launch on few workgroups behind a read-only pass is one of its store passes (a chunk of fewer
    // than 16 bytes has no such pass in front)
    c->in_store_pass = unpack && l.grid != 0 && c->pass.base != nullptr &&
                       p.packed >= c->pass.base && p.packed < c->pass.base + c->pass.bytes;
    if (unpack) {
        RunLaunch<true> run{&p, l.nblocks, HostMem{c}};
        return tp::dispatch_launch(l, p.nrd, run);
    }
    RunLaunch<false> run{&p, l.nblocks, HostMem{c}};
    return tp::dispatch_launch(l, p.nrd, run);
}

}  // namespace

extern "C" {

// Runs pack (unpack == 0) or unpack of `count` objects described by the StridedBlock
// (ndims, start, counts, strides) and `extent`, between host buffers:
//   typed  buffer [typed_buf, typed_buf + typed_len), objects' origin at typed_buf + origin
//   packed buffer [packed_buf, packed_buf + packed_len), data at packed_buf + position
// write_count (may be null) has one byte per byte of the destination buffer.
// result[0..2] = accesses out of bounds, unaligned accesses, destination bytes written again
// with a different value; result[3] = number of launches; result[4] = destination bytes written
// again with the same value.  `plan_text` receives the plan description.
// Returns a TP_* status from the planner, or 100 if a launch names no kernel variant.
int emul_transfer(int unpack, int ndims, int64_t start, const int64_t* counts, const int64_t* strides, int64_t extent,
                  int64_t count, char* typed_buf, int64_t typed_len, int64_t origin, char* packed_buf,
                  int64_t packed_len, int64_t position, int max_word_log2, int64_t max_rows_per_launch,
                  int64_t max_words_per_run, int allow_xpose, int stage, int64_t stage_bytes, uint8_t* write_count,
                  int64_t* result, char* plan_text, int64_t plan_text_len) {
    tp::PlanInput in;
    in.block.ndims = ndims;
    in.block.start = start;
    for (int d = 0; d < ndims; ++d) {
        in.block.counts[d] = counts[d];
        in.block.strides[d] = strides[d];
    }
    in.extent = extent;
    in.count = count;
    in.typed = typed_buf + origin;
    in.packed = packed_buf + position;
    in.unpack = unpack != 0;
    in.max_word_log2 = max_word_log2;
    in.max_rows_per_launch = max_rows_per_launch;
    in.max_words_per_run = max_words_per_run;
    in.allow_xpose = allow_xpose != 0;
    in.stage = stage;
    if (stage_bytes > 0) in.stage_bytes = stage_bytes;
    std::vector<tp::Launch> launches;
    const int rc = tp::plan_launches(in, &launches);
    if (rc != tp::kSuccess) return rc;
    if (plan_text && plan_text_len > 0) {
        const std::string text = tp::describe(launches);
        std::snprintf(plan_text, static_cast<size_t>(plan_text_len), "%s", text.c_str());
    }
    Checks c{typed_buf, typed_buf + typed_len, packed_buf, packed_buf + packed_len, write_count,
             unpack ? typed_buf : packed_buf};
    for (const tp::Launch& l : launches)
        if (!run_launch(l, unpack != 0, &c)) return 100;
    result[0] = c.oob;
    result[1] = c.unaligned;
    result[2] = c.rewritten;
    result[3] = static_cast<int64_t>(launches.size());
    result[4] = c.duplicates;
    result[5] = c.prefetched_hi - c.prefetched_lo;   // span of the packed bytes the read-only passes cover
    result[6] = c.misplaced;
    return 0;
}

// Plans a transfer without running it (no buffer is touched, so the shapes may be far larger than
// host memory): per launch, launches[4*i..] = tiles, workgroups the launch asks for, rows, kind.
// Returns the number of launches (filling at most `cap` of them), or minus a TP_* status.
int64_t emul_plan_only(int unpack, int ndims, int64_t start, const int64_t* counts, const int64_t* strides, int64_t extent,
                       int64_t count, int64_t typed_address, int64_t packed_address, int batched, int64_t* launches,
                       int64_t cap) {
    tp::PlanInput in;
    in.block.ndims = ndims;
    in.block.start = start;
    for (int d = 0; d < ndims; ++d) {
        in.block.counts[d] = counts[d];
        in.block.strides[d] = strides[d];
    }
    in.extent = extent;
    in.count = count;
    in.typed = reinterpret_cast<const char*>(static_cast<intptr_t>(typed_address));
    in.packed = reinterpret_cast<char*>(static_cast<intptr_t>(packed_address));
    in.unpack = unpack != 0;
    in.batched = batched != 0;
    std::vector<tp::Launch> planned;
    const int rc = tp::plan_launches(in, &planned);
    if (rc != tp::kSuccess) return -rc;
    std::vector<tp::Launch> singles = planned;
    std::vector<tp::BatchParams> batches;
    if (batched) {
        singles.clear();
        tp::make_batches(planned, &batches, &singles);
    }
    int64_t n = 0;
    auto put = [&](int64_t tiles, int64_t grid, int64_t rows, int64_t kind) {
        if (n < cap) {
            launches[4 * n] = tiles;
            launches[4 * n + 1] = grid;
            launches[4 * n + 2] = rows;
            launches[4 * n + 3] = kind;
        }
        ++n;
    };
    for (const tp::BatchParams& b : batches) put(b.nblocks, b.nblocks, 0, 100);
    for (const tp::Launch& l : singles) put(l.nblocks, l.grid ? l.grid : l.nblocks, l.kind == tp::kTile ? l.p.nrows : 0, l.kind);
    return n;
}

// Multiply-shift division (fastdiv.hpp) against the hardware divide: every divisor in
// [1, small_limit] with dividends around multiples of it and at the range ends, plus `random_pairs`
// pseudo-random (dividend < 2^31, divisor) pairs, powers of two included.  Returns the mismatches.
int64_t emul_fastdiv_mismatches(uint32_t small_limit, int64_t random_pairs, uint64_t seed) {
    int64_t bad = 0;
    auto check = [&bad](uint32_t n, const tp::FastDiv& f) {
        n &= 0x7fffffffu;
        if (tp::fastdiv(n, f) != n / f.divisor) ++bad;
    };
    for (uint32_t d = 1; d <= small_limit; ++d) {
        const tp::FastDiv f = tp::make_fastdiv(d);
        const uint32_t top = 0x7fffffffu / d * d;
        for (uint32_t n : {0u, 1u, d - 1, d, d + 1, 2 * d - 1, 2 * d, top - 1, top, top + 1, 0x7fffffffu, 0x7ffffffeu})
            check(n, f);
    }
    uint64_t x = seed | 1;
    auto next = [&x]() { x ^= x << 13; x ^= x >> 7; x ^= x << 17; return x; };
    for (int64_t k = 0; k < random_pairs; ++k) {
        uint32_t d = static_cast<uint32_t>(next() & 0x7fffffffu) | 1u;
        if (k % 3 == 0) d = 1u << (next() % 31);
        if (k % 3 == 1) d = (d % 70000u) + 1u;
        const tp::FastDiv f = tp::make_fastdiv(d);
        check(static_cast<uint32_t>(next()), f);
        check(0x7fffffffu, f);
        check(0x7fffffffu / d * d, f);
    }
    return bad;
}

// The batched form: n requests (request i: StridedBlock i, extent, object count, origin in the one
// typed buffer) sharing the packed buffer from `position` on.  Plans every request, groups the
// launches into batches exactly as the library does, and runs batch_thread for every workgroup
// and thread.  result[3] = number of batched launches, result[4] = launches left single,
// result[5] = destination bytes written again with the same value.
int emul_transfer_batch(int unpack, int n, const int* ndims, const int64_t* starts, const int64_t* counts,
                        const int64_t* strides, const int64_t* extents, const int64_t* objects,
                        const int64_t* origins, const int64_t* sizes, char* typed_buf, int64_t typed_len,
                        char* packed_buf, int64_t packed_len, int64_t position, uint8_t* write_count,
                        int64_t* result) {
    std::vector<tp::Launch> launches;
    int64_t pos = position;
    for (int i = 0; i < n; ++i) {
        tp::PlanInput in;
        in.block.ndims = ndims[i];
        in.block.start = starts[i];
        for (int d = 0; d < ndims[i]; ++d) {
            in.block.counts[d] = counts[i * tp::kMaxDims + d];
            in.block.strides[d] = strides[i * tp::kMaxDims + d];
        }
        in.extent = extents[i];
        in.count = objects[i];
        in.typed = typed_buf + origins[i];
        in.packed = packed_buf + pos;
        in.unpack = unpack != 0;
        in.batched = true;
        std::vector<tp::Launch> mine;
        const int rc = tp::plan_launches(in, &mine);
        if (rc != tp::kSuccess) return rc;
        launches.insert(launches.end(), mine.begin(), mine.end());
        pos += objects[i] * sizes[i];
    }
    std::vector<tp::BatchParams> batches;
    std::vector<tp::Launch> singles;
    tp::make_batches(launches, &batches, &singles);
    Checks c{typed_buf, typed_buf + typed_len, packed_buf, packed_buf + packed_len, write_count,
             unpack ? typed_buf : packed_buf};
    for (const tp::BatchParams& b : batches)
        for (uint32_t blk = 0; blk < b.nblocks; ++blk)
            for (uint32_t t = 0; t < static_cast<uint32_t>(tp::kBlockThreads); ++t) {
                if (unpack) tp::batch_thread<true>(b, blk, t, HostMem{&c});
                else tp::batch_thread<false>(b, blk, t, HostMem{&c});
            }
    for (const tp::Launch& l : singles)
        if (!run_launch(l, unpack != 0, &c)) return 100;
    result[0] = c.oob;
    result[1] = c.unaligned;
    result[2] = c.rewritten;
    result[3] = static_cast<int64_t>(batches.size());
    result[4] = static_cast<int64_t>(singles.size());
    result[5] = c.duplicates;
    return 0;
}

}  // extern "C"
