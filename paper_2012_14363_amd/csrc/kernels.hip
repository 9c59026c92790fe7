// Pack / unpack kernels for gfx950 (CDNA4, wave64).
//
// Pure data movement: the only arithmetic is address computation, so the design
// goal is to keep as many wide, coalesced memory accesses in flight as possible.
// One kernel template covers every StridedBlock:
//
//   * a workgroup of 256 threads is a flat tile of bx lanes along the contiguous
//     run times 256/bx rows (bx a power of two >= the run length in words, at most
//     256), so short runs still fill every wavefront with adjacent rows and the
//     contiguous side of the copy is written (pack) or read (unpack) as one dense
//     span per wavefront;
//   * each thread moves UX words along the run and UR rows, issuing all of its
//     loads before its first store;
//   * words sit at any byte address (unaligned vector accesses), and the last word of
//     a run is pulled back to end with the run, so neither addresses nor run lengths
//     restrict the word width;
//   * a row index is turned into its byte offset with multiply-shift division by
//     the (run-time constant) dimension counts; in the tiles for long runs the row
//     is uniform across the workgroup and that math runs on the scalar unit;
//   * all parameters arrive by value in the kernel-argument segment.
//
// Beside it: the transposing kernel (tiles through LDS), the batched kernel (many
// planned launches as one grid) and the read-only pass of a staged unpack, which
// brings packed bytes into L2 ahead of the stores that consume them.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kernels.hpp"
#include "tile_body.hpp"

namespace tp {

namespace {

// Memory accesses with a streaming hint.  Every byte is touched once, so loads and
// stores can carry the non-temporal bit (`nt`): the data then does not displace
// other lines in L2 / Infinity Cache.  NT bit 0: loads, bit 1: stores, bit 2: stores
// also carry `sc1`, which has L2 write them through at once instead of holding the
// line until something evicts it.
// The word is accessed through a type of alignment 1: the address may be any byte, and
// the compiler, which knows that this target takes unaligned accesses, still emits one
// global_load/store of the full width.
template <int NT>
struct DeviceMem {
    template <class W>
    __device__ __forceinline__ W load(const char* p) const {
        typedef W Unaligned __attribute__((aligned(1)));
        if constexpr (NT & 1) return __builtin_nontemporal_load(reinterpret_cast<const Unaligned*>(p));
        else return *reinterpret_cast<const Unaligned*>(p);
    }
    template <class W>
    __device__ __forceinline__ void store(char* p, const W& v) const {
        typedef W Unaligned __attribute__((aligned(1)));
        if constexpr (NT & 4) store_through(p, v);
        else if constexpr (NT & 2) __builtin_nontemporal_store(v, reinterpret_cast<Unaligned*>(p));
        else *reinterpret_cast<Unaligned*>(p) = v;
    }
    // Keeps a loaded value alive without using it (prefetch passes).
    template <class W>
    __device__ __forceinline__ void consume(const W& v) const {
        asm volatile("" : : "v"(v));
    }
    // `global_store ... sc1 nt`.  No builtin sets both bits, hence the instruction by hand; like the
    // plain store it takes any byte address.  After a store of more than 8 bytes the next vector
    // instruction must not overwrite the data registers; the compiler spaces the stores it emits
    // itself but cannot see into this one, so an s_nop follows the 16-byte form.
    template <class W>
    __device__ __forceinline__ static void store_through(char* p, const W& v) {
        if constexpr (sizeof(W) == 1)
            asm volatile("global_store_byte %0, %1, off sc1 nt" : : "v"(p), "v"(static_cast<uint32_t>(v)) : "memory");
        else if constexpr (sizeof(W) == 2)
            asm volatile("global_store_short %0, %1, off sc1 nt" : : "v"(p), "v"(static_cast<uint32_t>(v)) : "memory");
        else if constexpr (sizeof(W) == 4)
            asm volatile("global_store_dword %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
        else if constexpr (sizeof(W) == 8)
            asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
        else
            asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 0" : : "v"(p), "v"(v) : "memory");
    }
};

template <int WLOG2, int UX, int UR, bool UNPACK, int NRD, int NT>
__global__ void __launch_bounds__(kBlockThreads) tile_kernel(const KParams p) {
    // one workgroup per tile, or (staged unpack) fewer workgroups that each take every gridDim.x-th tile
    for (uint32_t tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x)
        tile_thread<WLOG2, UX, UR, UNPACK, NRD>(p, tile, threadIdx.x, DeviceMem<NT>{});
}

// Read-only pass of a staged unpack: plain (cached) loads, so the bytes stay in this XCD's L2.
__global__ void __launch_bounds__(kBlockThreads) prefetch_kernel(const PrefetchParams f) {
    prefetch_thread(f, blockIdx.x, gridDim.x, threadIdx.x, DeviceMem<0>{});
}

// Transposing tiles through LDS (tile_body.hpp: xpose_phase).
template <int WLOG2, bool UNPACK, bool SQUARE>
__global__ void __launch_bounds__(kBlockThreads) xpose_kernel(const XParams p) {
    using W = typename WordOf<WLOG2>::type;
    __shared__ W lds[XposeTile<WLOG2>::kLdsWords];
    xpose_phase<WLOG2, UNPACK, true, SQUARE>(p, blockIdx.x, threadIdx.x, DeviceMem<3>{}, lds);
    __syncthreads();
    xpose_phase<WLOG2, UNPACK, false, SQUARE>(p, blockIdx.x, threadIdx.x, DeviceMem<3>{}, lds);
}

template <int WLOG2, bool UNPACK>
void launch_xpose(const Launch& l, hipStream_t stream) {
    const dim3 grid(l.nblocks), block(kBlockThreads);
    if (xpose_is_square(l.x, WLOG2)) hipLaunchKernelGGL((xpose_kernel<WLOG2, UNPACK, true>), grid, block, 0, stream, l.x);
    else hipLaunchKernelGGL((xpose_kernel<WLOG2, UNPACK, false>), grid, block, 0, stream, l.x);
}

template <bool UNPACK>
hipError_t enqueue_xpose(const Launch& l, hipStream_t stream) {
    // what the kernel's lane mapping and LDS tile assume of their parameters
    const XParams& x = l.x;
    if (x.ew == 0 || x.te_a == 0 || x.te_b == 0 || x.fa_log2 > 8 || x.fb_log2 > 8 ||
        x.pitch < x.te_a * x.ew || uint64_t{x.te_b} * x.pitch > static_cast<uint64_t>(xpose_lds_words(l.word_log2)))
        return hipErrorInvalidValue;
    switch (l.word_log2) {
    case 0: launch_xpose<0, UNPACK>(l, stream); break;
    case 1: launch_xpose<1, UNPACK>(l, stream); break;
    case 2: launch_xpose<2, UNPACK>(l, stream); break;
    case 3: launch_xpose<3, UNPACK>(l, stream); break;
    case 4: launch_xpose<4, UNPACK>(l, stream); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Many planned launches, of different datatypes, as one grid: a workgroup looks up
// the descriptor that owns it (binary search over at most 40 block ranges, scalar)
// and runs the same tile body.  Saves one launch per datatype where launches are
// short, e.g. the 26 regions of a halo exchange.
template <bool UNPACK>
__global__ void __launch_bounds__(kBlockThreads) batch_kernel(const BatchParams b) {
    batch_thread<UNPACK>(b, blockIdx.x, threadIdx.x, DeviceMem<3>{});
}

using KernelFn = void (*)(const KParams);

// Visitor for dispatch_launch: the kernel instantiation a launch names.
template <bool UNPACK>
struct PickKernel {
    int nt = 3;
    KernelFn fn = nullptr;
    template <int WLOG2, int UX, int UR, int NRD>
    void operator()() {
        switch (nt) {
        case 0: fn = tile_kernel<WLOG2, UX, UR, UNPACK, NRD, 0>; break;
        case 1: fn = tile_kernel<WLOG2, UX, UR, UNPACK, NRD, 1>; break;
        case 2: fn = tile_kernel<WLOG2, UX, UR, UNPACK, NRD, 2>; break;
        case 3: fn = tile_kernel<WLOG2, UX, UR, UNPACK, NRD, 3>; break;
        case 6: fn = tile_kernel<WLOG2, UX, UR, UNPACK, NRD, 6>; break;
        case 7: fn = tile_kernel<WLOG2, UX, UR, UNPACK, NRD, 7>; break;
        default: break;
        }
    }
};

}  // namespace

hipError_t enqueue(const Launch& l, bool unpack, hipStream_t stream) {
    if (l.nblocks == 0 || l.grid > l.nblocks || (l.grid ? l.grid : l.nblocks) > kMaxGrid) return hipErrorInvalidValue;
    const dim3 grid(l.grid ? l.grid : l.nblocks), block(kBlockThreads);
    if (l.kind == kXpose) {
        if (l.grid) return hipErrorInvalidValue;
        return unpack ? enqueue_xpose<true>(l, stream) : enqueue_xpose<false>(l, stream);
    }
    if (l.kind == kPrefetch) {
        // what prefetch_thread assumes of its parameters
        const PrefetchParams& f = l.f;
        if (!f.base || f.bytes < 16 || f.tile_bytes < 16 || (f.tile_bytes & (f.tile_bytes - 1)) || f.ntiles != l.nblocks ||
            (f.bytes + f.tile_bytes - 1) / f.tile_bytes != f.ntiles)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL(prefetch_kernel, grid, block, 0, stream, f);
        return hipGetLastError();
    }
    const KParams p = kernel_params(l);
    KernelFn fn = nullptr;
    if (unpack) {
        PickKernel<true> pick;
        pick.nt = l.nt;
        if (dispatch_launch(l, p.nrd, pick)) fn = pick.fn;
    } else {
        PickKernel<false> pick;
        pick.nt = l.nt;
        if (dispatch_launch(l, p.nrd, pick)) fn = pick.fn;
    }
    if (!fn) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fn, grid, block, 0, stream, p);
    return hipGetLastError();
}

hipError_t enqueue_batch(const BatchParams& b, bool unpack, hipStream_t stream) {
    if (b.n == 0 || b.nblocks == 0 || b.nblocks > kMaxGrid) return hipErrorInvalidValue;
    if (unpack) hipLaunchKernelGGL(batch_kernel<true>, dim3(b.nblocks), dim3(kBlockThreads), 0, stream, b);
    else hipLaunchKernelGGL(batch_kernel<false>, dim3(b.nblocks), dim3(kBlockThreads), 0, stream, b);
    return hipGetLastError();
}

}  // namespace tp
