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
template <int NRD>
TP_HD inline int64_t row_offset(uint32_t r, const KParams& p) {
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
template <int WLOG2, int UX, int UR, bool UNPACK, int NRD, class Mem>
TP_HD inline void tile_thread(const KParams& p, uint32_t block, uint32_t tid, Mem mem) {
    using W = typename WordOf<WLOG2>::type;
    const uint32_t tx = tid & ((1u << p.bx_log2) - 1u);
    const uint32_t tr = tid >> p.bx_log2;
    const uint32_t br = static_cast<uint32_t>(kBlockThreads) >> p.bx_log2;
    const uint32_t rc = fastdiv(block, p.xc_div);
    const uint32_t xc = block - rc * p.nxc;
    const uint32_t x0 = ((xc * UX) << p.bx_log2) + tx;
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
            const uint32_t x = x0 + (static_cast<uint32_t>(ux) << p.bx_log2);
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
