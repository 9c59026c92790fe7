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
// of each of UR rows.  `Mem` supplies load/store of words at any byte address (plain,
// possibly unaligned accesses on the device).
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
            // the last word of a run ends with the run (it overlaps the word before it if the
            // run length is no multiple of the word)
            const int64_t xb = (static_cast<int64_t>(x) << WLOG2) - (x + 1u == p.n0 ? p.tail_back : 0u);
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

// Thread `tid` of workgroup `block` of `nblocks` in a read-only pass.  The workgroup owns tiles
// block, block + nblocks, ...; its threads walk the 16-byte words of all of them as one list, four
// loads in flight per thread, and drop the values.  The last word ends with the bytes (they are
// at least 16).  tile_bytes is a power of two (>= 16), so the list index splits with a shift.
template <class Mem>
TP_HD inline void prefetch_thread(const PrefetchParams& f, uint32_t block, uint32_t nblocks, uint32_t tid, Mem mem) {
    if (block >= f.ntiles) return;
    uint32_t wlog = 0;
    while ((16u << wlog) < f.tile_bytes) ++wlog;                  // words per tile = 1 << wlog
    const uint64_t my_tiles = (static_cast<uint64_t>(f.ntiles) - block + nblocks - 1) / nblocks;
    const uint64_t words = my_tiles << wlog;
    constexpr int kInFlight = 4;
    for (uint64_t first = tid; first < words; first += static_cast<uint64_t>(kBlockThreads) * kInFlight) {
        Word16 v[kInFlight];
        bool ok[kInFlight];
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            const uint64_t idx = first + static_cast<uint64_t>(k) * kBlockThreads;
            const uint64_t tile = block + (idx >> wlog) * nblocks;
            const uint64_t off = tile * f.tile_bytes + ((idx & ((uint64_t{1} << wlog) - 1)) << 4);
            ok[k] = idx < words && off < f.bytes;
            const uint64_t at = off + 16 <= f.bytes ? off : f.bytes - 16;
            if (ok[k]) v[k] = mem.template load<Word16>(f.base + at);
        }
#pragma unroll
        for (int k = 0; k < kInFlight; ++k)
            if (ok[k]) mem.consume(v[k]);
    }
}

// ------------------------------------------------------------------ transposing tiles
template <int WLOG2>
struct XposeTile {
    static constexpr int kLdsWords = xpose_lds_words(WLOG2);  // te_b rows of `pitch` words at most
};

// Where workgroup `block` works: its tile's first element along A and B and the byte offsets of
// the tile's outer position on both sides.
struct XposeOrigin {
    uint32_t a0, b0;
    int64_t typed_off, packed_off;
};

TP_HD inline XposeOrigin xpose_origin(const XParams& p, uint32_t block) {
    uint32_t q = fastdiv(block, p.tiles_a_div);
    const uint32_t ta = block - q * p.tiles_a;
    uint32_t o = fastdiv(q, p.tiles_b_div);
    const uint32_t tb = q - o * p.tiles_b;
    XposeOrigin g;
    g.a0 = ta * p.te_a;
    g.b0 = tb * p.te_b;
    g.typed_off = 0;
    g.packed_off = 0;
    for (uint32_t d = 0; d < p.nod; ++d) {
        const uint32_t nq = d + 1 < p.nod ? fastdiv(o, p.odiv[d]) : 0u;
        const uint32_t i = d + 1 < p.nod ? o - nq * p.ocount[d] : o;
        g.typed_off += static_cast<int64_t>(i) * p.otstride[d];
        g.packed_off += static_cast<int64_t>(i) * p.opstride[d];
        o = nq;
    }
    return g;
}

// Word `w` of element (a, b) of the tile's outer position, on the typed and on the packed side.
template <int WLOG2>
TP_HD inline const char* xpose_typed(const XParams& p, const XposeOrigin& g, uint32_t a, uint32_t b, uint32_t w) {
    return p.strided + g.typed_off + static_cast<int64_t>(b) * p.tb_stride +
           (static_cast<int64_t>(static_cast<uint64_t>(a) * p.ew + w) << WLOG2);
}
template <int WLOG2>
TP_HD inline char* xpose_packed(const XParams& p, const XposeOrigin& g, uint32_t a, uint32_t b, uint32_t w) {
    return p.packed + g.packed_off + static_cast<int64_t>(a) * p.pa_stride +
           (static_cast<int64_t>(static_cast<uint64_t>(b) * p.ew + w) << WLOG2);
}

// One phase of thread `tid`.  LOAD: read the tile from the source side into LDS; else write it from
// LDS to the destination side.  Lanes run along the dimension that is contiguous on that side (A
// on the typed side, B on the packed side), one word each; the tile lives in LDS as
// lds[b * pitch + a * ew + w].  The second phase may only start when every thread of the workgroup
// has finished the first.
// SQUARE: the common case of one-word elements in full square tiles (te_a == te_b ==
// xpose_fast_words, pitch one more), with those parameters as compile-time constants.
template <int WLOG2, bool UNPACK, bool LOAD, bool SQUARE, class Mem>
TP_HD inline void xpose_phase(const XParams& p, uint32_t block, uint32_t tid, Mem mem,
                              typename WordOf<WLOG2>::type* lds) {
    using W = typename WordOf<WLOG2>::type;
    const XposeOrigin g = xpose_origin(p, block);
    // the typed side is this phase's side when packing and loading, or unpacking and storing
    constexpr bool kTypedSide = UNPACK != LOAD;
    constexpr uint32_t kEdge = static_cast<uint32_t>(xpose_fast_words(WLOG2));
    constexpr uint32_t kEdgeLog2 = kEdge == 32 ? 5u : kEdge == 64 ? 6u : 7u;
    const uint32_t ew = SQUARE ? 1u : p.ew, pitch = SQUARE ? kEdge + 1u : p.pitch;
    const uint32_t f_log2 = SQUARE ? kEdgeLog2 : kTypedSide ? p.fa_log2 : p.fb_log2;
    const uint32_t te_fast = SQUARE ? kEdge : kTypedSide ? p.te_a : p.te_b;
    const uint32_t te_slow = SQUARE ? kEdge : kTypedSide ? p.te_b : p.te_a;
    const uint32_t rows_per_pass = static_cast<uint32_t>(kBlockThreads) >> f_log2;
    const uint32_t lanes = 1u << f_log2, slow0 = tid >> f_log2;
    // Tile rows longer than the lanes along them (thin tiles grown along the other dimension) are
    // walked in chunks of `lanes` words.
    for (uint32_t fast = tid & (lanes - 1u); fast < te_fast * ew; fast += lanes) {
        const uint32_t fe = ew == 1 ? fast : fast / ew;  // element and word within it along the fast dimension
        const uint32_t fw = fast - fe * ew;
        // Tile rows in groups of kGroup: all of a group's loads are issued before its first store,
        // so that many memory accesses are in flight per thread.
        constexpr uint32_t kGroup = 16;
        for (uint32_t first = slow0; first < te_slow; first += kGroup * rows_per_pass) {
            W v[kGroup];
            bool ok[kGroup];
            W* cell[kGroup];
            char* far[kGroup];
#pragma unroll
            for (uint32_t k = 0; k < kGroup; ++k) {
                const uint32_t slow = first + k * rows_per_pass;
                const uint32_t la = kTypedSide ? fe : slow, lb = kTypedSide ? slow : fe;
                const uint32_t a = g.a0 + la, b = g.b0 + lb;
                ok[k] = slow < te_slow && a < p.ca && b < p.cb;
                // lanes with nothing to move address the tile's first element, which always exists
                const uint32_t sa = ok[k] ? a : g.a0, sb = ok[k] ? b : g.b0, sw = ok[k] ? fw : 0u;
                cell[k] = lds + (ok[k] ? lb * pitch + la * ew + fw : 0u);
                far[k] = kTypedSide ? const_cast<char*>(xpose_typed<WLOG2>(p, g, sa, sb, sw)) : xpose_packed<WLOG2>(p, g, sa, sb, sw);
                if (LOAD) v[k] = mem.template load<W>(far[k]);
                else if (ok[k]) v[k] = *cell[k];
            }
#pragma unroll
            for (uint32_t k = 0; k < kGroup; ++k) {
                if (!ok[k]) continue;
                if (LOAD) *cell[k] = v[k];
                else mem.template store<W>(far[k], v[k]);
            }
        }
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
        if (ux == 1 && ur == 1) return by_nrd(w, I1{}, I1{});
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
    uint32_t n0, nrows, bx_log2, nxc, nrd, tail_back;
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
    p.tail_back = d.tile >> 4;
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
    const uint32_t wl = b.d[j].word_log2, tile = b.d[j].tile & 3u, nrd = b.d[j].nrd;
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
// f.template operator()<WLOG2, UX, UR, NRD>().  Shared by the device launcher and by the host
// emulation the tests run, so a wrong mapping shows up on the CPU.
template <class F>
inline bool dispatch_launch(const Launch& l, uint32_t nrd, F&& f) {
    return dispatch_variant(l.word_log2, l.ux, l.ur, nrd, f);
}

// A launch as the kernel sees it: a single row gets one dummy row dimension so the
// unrolled, division-free variant serves it.
inline KParams kernel_params(const Launch& l) {
    KParams p = l.p;
    p.ntiles = l.nblocks;
    if (p.nrd == 0) {
        p.nrd = 1;
        p.rcount[0] = 1;
        p.rstride[0] = 0;
        p.rdiv[0] = make_fastdiv(1);
    }
    return p;
}

}  // namespace tp
