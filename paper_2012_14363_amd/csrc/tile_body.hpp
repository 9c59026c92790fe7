// The per-thread body of the tile kernel, written once for the device and for a
// host build: tests compile it with the host compiler and run every planned
// launch thread by thread under bounds checks before anything goes to a GPU.
#pragma once

#include <cstdint>
#include <type_traits>

#include "fastdiv.hpp"
#include "plan.hpp"

namespace tp {

// 16-byte access word: a native vector type so one global_load/store_dwordx4 moves it.
#if defined(__clang__)
typedef uint32_t Word16 __attribute__((ext_vector_type(4)));
#else
typedef uint32_t Word16 __attribute__((vector_size(16)));
#endif

template <int LOG2>
struct WordOf;
template <>
struct WordOf<0> { using type = uint8_t; };
template <>
struct WordOf<1> { using type = uint16_t; };
template <>
struct WordOf<2> { using type = uint32_t; };
template <>
struct WordOf<3> { using type = uint64_t; };
template <>
struct WordOf<4> { using type = Word16; };

// Byte offset of row r in the typed buffer.  NRD > 0: that many row dimensions,
// unrolled; NRD == 0: p.nrd (>= 1) of them, looped.
template <int NRD, class P>
TP_HD inline int64_t row_offset(uint32_t r, const P& p) {
    int64_t off = 0;
    const int n = NRD > 0 ? NRD : static_cast<int>(p.nrd);
#pragma unroll
    for (int d = 0; d < n - 1; ++d) {
        const uint32_t q = fastdiv(r, p.rdiv[d]);
        const uint32_t i = r - q * p.rcount[d];
        off += static_cast<int64_t>(i) * p.rstride[d];
        r = q;
    }
    off += static_cast<int64_t>(r) * p.rstride[n - 1];
    return off;
}

// Thread `tid` of workgroup `block`.  The workgroup is a flat tile of
// bx = 1 << bx_log2 lanes along the run by 256/bx rows; this thread moves UX words
// of each of UR rows.  `Mem` supplies load/store (plain accesses on the device).
// `P` is KParams, or the register-resident SmallParams a batched launch unpacks.
template <int WLOG2, int UX, int UR, bool UNPACK, int NRD, class P, class Mem>
TP_HD inline void tile_thread(const P& p, uint32_t block, uint32_t tid, Mem mem) {
    using W = typename WordOf<WLOG2>::type;
    // Tiles that move more than one word per thread along the run are only planned for runs
    // longer than the workgroup (bx == 256): every thread is then on the same row, the row
    // index depends on the workgroup id alone and its arithmetic stays on the scalar unit.
    constexpr bool kWholeGroupOnOneRow = UX > 1;
    const uint32_t bx_log2 = kWholeGroupOnOneRow ? 8u : p.bx_log2;
    const uint32_t tx = kWholeGroupOnOneRow ? tid : tid & ((1u << bx_log2) - 1u);
    const uint32_t tr = kWholeGroupOnOneRow ? 0u : tid >> bx_log2;
    const uint32_t br = static_cast<uint32_t>(kBlockThreads) >> bx_log2;
    const uint32_t rc = fastdiv(block, p.xc_div);
    const uint32_t xc = block - rc * p.nxc;
    const uint32_t x0 = ((xc * UX) << bx_log2) + tx;
    const uint32_t r0 = rc * (br * UR) + tr;

    const char* src[UR][UX];
    char* dst[UR][UX];
    bool ok[UR][UX];
#pragma unroll
    for (int ur = 0; ur < UR; ++ur) {
        const uint32_t r = r0 + ur * br;
        const bool row_ok = r < p.nrows;
        const uint32_t rr = row_ok ? r : 0u;
        const int64_t soff = row_offset<NRD>(rr, p);
        const int64_t poff = static_cast<int64_t>(rr) * p.row_pitch;
#pragma unroll
        for (int ux = 0; ux < UX; ++ux) {
            const uint32_t x = x0 + (static_cast<uint32_t>(ux) << bx_log2);
            ok[ur][ux] = row_ok && x < p.n0;
            const int64_t xb = static_cast<int64_t>(x) << WLOG2;
            const char* s = p.strided + soff + xb;
            char* q = p.packed + poff + xb;
            src[ur][ux] = UNPACK ? q : s;
            dst[ur][ux] = UNPACK ? const_cast<char*>(s) : q;
        }
    }
    W v[UR][UX];
#pragma unroll
    for (int ur = 0; ur < UR; ++ur)
#pragma unroll
        for (int ux = 0; ux < UX; ++ux)
            if (ok[ur][ux]) v[ur][ux] = mem.template load<W>(src[ur][ux]);
#pragma unroll
    for (int ur = 0; ur < UR; ++ur)
#pragma unroll
        for (int ux = 0; ux < UX; ++ux)
            if (ok[ur][ux]) mem.template store<W>(dst[ur][ux], v[ur][ux]);
}

// ------------------------------------------------------------------ shifted copy
// Runs whose source and destination are not aligned alike (odd addresses, odd run lengths)
// would otherwise move byte by byte.  Here the destination row is cut into a head of bytes up
// to its first 4-byte boundary, whole aligned 4-byte words, and a tail of bytes.  Lane
// x < nb builds destination word x from the two aligned source words that straddle it (a
// funnel shift by the rows' relative misalignment) and stores it aligned; lane x == nb copies
// the head and tail bytes.  Every store is exact: no byte outside the run is written.  A
// source load may cover bytes outside the run, but always inside an aligned word that also
// holds a byte of the run, hence inside a mapped page.
TP_HD inline uint32_t funnel_shift_bytes(uint32_t lo, uint32_t hi, uint32_t bytes) {
    return static_cast<uint32_t>(((static_cast<uint64_t>(hi) << 32) | lo) >> (8u * bytes));
}

template <int UX, int UR, bool UNPACK, int NRD, class P, class Mem>
TP_HD inline void shift_thread(const P& p, uint32_t block, uint32_t tid, Mem mem) {
    // 4-byte words: measured faster than 16-byte words here (31 vs 42 us for 64 MiB), and as fast
    // as any width in the plain tile kernel
    constexpr int WLOG2 = 2;
    using W = uint32_t;
    constexpr uint32_t kWordBytes = 1u << WLOG2;
    constexpr bool kWholeGroupOnOneRow = UX > 1;
    const uint32_t bx_log2 = kWholeGroupOnOneRow ? 8u : p.bx_log2;
    const uint32_t tx = kWholeGroupOnOneRow ? tid : tid & ((1u << bx_log2) - 1u);
    const uint32_t tr = kWholeGroupOnOneRow ? 0u : tid >> bx_log2;
    const uint32_t br = static_cast<uint32_t>(kBlockThreads) >> bx_log2;
    const uint32_t rc = fastdiv(block, p.xc_div);
    const uint32_t xc = block - rc * p.nxc;
    const uint32_t x0 = ((xc * UX) << bx_log2) + tx;
    const uint32_t r0 = rc * (br * UR) + tr;
    const uint32_t len = p.run_len;

    const char* src_word[UR][UX];  // aligned source word holding the destination word's first byte
    char* dst_word[UR][UX];
    uint32_t shift[UR];
    int role[UR][UX];  // 0: idle, 1: whole word, 2: head and tail bytes
    const char* src_row[UR];
    char* dst_row[UR];
    uint32_t head[UR], body_words[UR];
#pragma unroll
    for (int ur = 0; ur < UR; ++ur) {
        const uint32_t r = r0 + ur * br;
        const bool row_ok = r < p.nrows;
        const uint32_t rr = row_ok ? r : 0u;
        const char* s = p.strided + row_offset<NRD>(rr, p);
        char* q = p.packed + static_cast<int64_t>(rr) * p.row_pitch;
        src_row[ur] = UNPACK ? q : s;
        dst_row[ur] = UNPACK ? const_cast<char*>(s) : q;
        const uint32_t to_boundary =
            static_cast<uint32_t>(-reinterpret_cast<uintptr_t>(dst_row[ur])) & (kWordBytes - 1u);
        head[ur] = to_boundary < len ? to_boundary : len;
        body_words[ur] = (len - head[ur]) >> WLOG2;
        const uintptr_t first = reinterpret_cast<uintptr_t>(src_row[ur]) + head[ur];
        shift[ur] = static_cast<uint32_t>(first & (kWordBytes - 1u));
#pragma unroll
        for (int ux = 0; ux < UX; ++ux) {
            const uint32_t x = x0 + (static_cast<uint32_t>(ux) << bx_log2);
            role[ur][ux] = !row_ok ? 0 : x < body_words[ur] ? 1 : x == body_words[ur] ? 2 : 0;
            const int64_t xb = static_cast<int64_t>(x) << WLOG2;
            src_word[ur][ux] = src_row[ur] + head[ur] - shift[ur] + xb;
            dst_word[ur][ux] = dst_row[ur] + head[ur] + xb;
        }
    }
    // Loads are unconditional so that all of a thread's loads are in flight together: lanes
    // with no word to move, and the second load of a row that needs no shift, re-read an address
    // that is always valid - the aligned word holding the run's first byte.
    W lo[UR][UX], hi[UR][UX];
#pragma unroll
    for (int ur = 0; ur < UR; ++ur) {
        const char* safe = src_row[ur] - (reinterpret_cast<uintptr_t>(src_row[ur]) & (kWordBytes - 1u));
#pragma unroll
        for (int ux = 0; ux < UX; ++ux) {
            const char* first = role[ur][ux] == 1 ? src_word[ur][ux] : safe;
            const char* second = (role[ur][ux] == 1 && shift[ur] != 0u) ? src_word[ur][ux] + kWordBytes : first;
            lo[ur][ux] = mem.template load_straddling<W>(first);
            hi[ur][ux] = mem.template load_straddling<W>(second);
        }
    }
#pragma unroll
    for (int ur = 0; ur < UR; ++ur)
#pragma unroll
        for (int ux = 0; ux < UX; ++ux)
            if (role[ur][ux] == 1)
                mem.template store<W>(dst_word[ur][ux], funnel_shift_bytes(lo[ur][ux], hi[ur][ux], shift[ur]));
    // ragged ends, one lane per row
#pragma unroll
    for (int ur = 0; ur < UR; ++ur)
#pragma unroll
        for (int ux = 0; ux < UX; ++ux)
            if (role[ur][ux] == 2) {
                for (uint32_t k = 0; k < head[ur]; ++k)
                    mem.template store<uint8_t>(dst_row[ur] + k, mem.template load<uint8_t>(src_row[ur] + k));
                for (uint32_t k = head[ur] + (body_words[ur] << WLOG2); k < len; ++k)
                    mem.template store<uint8_t>(dst_row[ur] + k, mem.template load<uint8_t>(src_row[ur] + k));
            }
}

// Calls f.template operator()<WLOG2, UX, UR, NRD>() for the variant a launch names;
// returns false if there is none.  nrd 0 and 1 share the division-free variant
// (the caller gives a single row one dummy dimension).
template <class F>
inline bool dispatch_variant(int word_log2, int ux, int ur, uint32_t nrd, F&& f) {
    auto by_nrd = [&](auto w, auto x, auto r) {
        constexpr int WL = decltype(w)::value, X = decltype(x)::value, R = decltype(r)::value;
        if (nrd <= 1) f.template operator()<WL, X, R, 1>();
        else if (nrd == 2) f.template operator()<WL, X, R, 2>();
        else f.template operator()<WL, X, R, 0>();
        return true;
    };
    auto by_tile = [&](auto w) {
        using I1 = std::integral_constant<int, 1>;
        using I2 = std::integral_constant<int, 2>;
        using I4 = std::integral_constant<int, 4>;
        if (ux == 4 && ur == 1) return by_nrd(w, I4{}, I1{});
        if (ux == 2 && ur == 2) return by_nrd(w, I2{}, I2{});
        if (ux == 1 && ur == 4) return by_nrd(w, I1{}, I4{});
        return false;
    };
    switch (word_log2) {
    case 0: return by_tile(std::integral_constant<int, 0>{});
    case 1: return by_tile(std::integral_constant<int, 1>{});
    case 2: return by_tile(std::integral_constant<int, 2>{});
    case 3: return by_tile(std::integral_constant<int, 3>{});
    case 4: return by_tile(std::integral_constant<int, 4>{});
    default: return false;
    }
}

// ------------------------------------------------------------------ batched launches
// One descriptor of a batched launch, unpacked from its compact kernel-argument
// form into the field names tile_thread reads.  At most kBatchRowDims row
// dimensions, all indexed with compile-time constants, so it lives in registers.
struct SmallParams {
    const char* strided;
    char* packed;
    int64_t row_pitch;
    uint32_t n0, nrows, bx_log2, nxc, nrd;
    FastDiv xc_div;
    FastDiv rdiv[kBatchRowDims];
    uint32_t rcount[kBatchRowDims];
    int64_t rstride[kBatchRowDims];
};

TP_HD inline SmallParams unpack_desc(const BatchDesc& d) {
    SmallParams p;
    p.strided = d.strided;
    p.packed = d.packed;
    p.row_pitch = d.row_pitch;
    p.n0 = d.n0;
    p.nrows = d.nrows;
    p.bx_log2 = d.bx_log2;
    p.nxc = d.nxc;
    p.nrd = d.nrd;
    p.xc_div.mul = d.xc_mul;
    p.xc_div.shift = d.xc_shift;
    p.xc_div.divisor = d.nxc;
    for (int k = 0; k < kBatchRowDims; ++k) {
        p.rdiv[k].mul = d.rmul[k];
        p.rdiv[k].shift = d.rshift[k];
        p.rdiv[k].divisor = d.rcount[k];
        p.rcount[k] = d.rcount[k];
        p.rstride[k] = d.rstride[k];
    }
    return p;
}

// Index of the descriptor that owns workgroup `block`: the first j with block < block_end[j].
TP_HD inline uint32_t find_desc(const BatchParams& b, uint32_t block) {
    uint32_t lo = 0, hi = b.n - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (block < b.block_end[mid]) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Workgroup `block`, thread `tid` of a batched launch: find the descriptor, then run the
// tile body of the variant it names (word width x tile x row dimensions, all unrolled).
template <bool UNPACK, class Mem>
TP_HD inline void batch_thread(const BatchParams& b, uint32_t block, uint32_t tid, Mem mem) {
    const uint32_t j = find_desc(b, block);
    const uint32_t first = j == 0 ? 0u : b.block_end[j - 1];
    const SmallParams p = unpack_desc(b.d[j]);
    const uint32_t local = block - first;
    const uint32_t wl = b.d[j].word_log2, tile = b.d[j].tile, nrd = b.d[j].nrd;
#define TP_BATCH_CASE(WL, X, R, N) tile_thread<WL, X, R, UNPACK, N>(p, local, tid, mem)
#define TP_BATCH_NRD(WL, X, R)            \
    do {                                  \
        if (nrd <= 1) TP_BATCH_CASE(WL, X, R, 1);      \
        else if (nrd == 2) TP_BATCH_CASE(WL, X, R, 2); \
        else TP_BATCH_CASE(WL, X, R, 3);               \
    } while (0)
#define TP_BATCH_TILE(WL)                              \
    do {                                               \
        if (tile == 0) TP_BATCH_NRD(WL, 1, 4);         \
        else if (tile == 1) TP_BATCH_NRD(WL, 2, 2);    \
        else TP_BATCH_NRD(WL, 4, 1);                   \
    } while (0)
    switch (wl) {
    case 0: TP_BATCH_TILE(0); break;
    case 1: TP_BATCH_TILE(1); break;
    case 2: TP_BATCH_TILE(2); break;
    case 3: TP_BATCH_TILE(3); break;
    default: TP_BATCH_TILE(4); break;
    }
#undef TP_BATCH_TILE
#undef TP_BATCH_NRD
#undef TP_BATCH_CASE
}

// The one place that maps a planned launch to the kernel variant that runs it: calls
// f.template operator()<KIND, WLOG2, UX, UR, NRD>().  Shared by the device launcher and by the
// host emulation the tests run, so a wrong mapping shows up on the CPU.
template <int KIND, class F>
struct KindOf {
    F& f;
    template <int WLOG2, int UX, int UR, int NRD>
    void operator()() {
        f.template operator()<KIND, WLOG2, UX, UR, NRD>();
    }
};

template <class F>
inline bool dispatch_launch(const Launch& l, uint32_t nrd, F&& f) {
    if (l.kind == kShift) {
        KindOf<kShift, std::remove_reference_t<F>> k{f};
        return l.word_log2 == 2 && dispatch_variant(2, l.ux, l.ur, nrd, k);
    }
    KindOf<kTile, std::remove_reference_t<F>> k{f};
    return dispatch_variant(l.word_log2, l.ux, l.ur, nrd, k);
}

// A launch as the kernel sees it: a single row gets one dummy row dimension so the
// unrolled, division-free variant serves it.
inline KParams kernel_params(const Launch& l) {
    KParams p = l.p;
    if (p.nrd == 0) {
        p.nrd = 1;
        p.rcount[0] = 1;
        p.rstride[0] = 0;
        p.rdiv[0] = make_fastdiv(1);
    }
    return p;
}

}  // namespace tp
