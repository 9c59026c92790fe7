// Call-time planning (paper Sec. 3.3, "Kernel Selection"): from a committed type's
// StridedBlock plus what is only known at the call - object count, buffer
// addresses - to a list of kernel launches with all parameters by value.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "fastdiv.hpp"
#include "strided_block.hpp"

namespace tp {

constexpr int kBlockThreads = 256;  // four wave64 per workgroup
// The runtime launches no grid of 2^32 threads or more: with 256-thread workgroups a launch has at
// most 2^24 - 1 of them.  Launches of more tiles run on that many workgroups, each taking every
// gridDim.x-th tile; launches whose kernels take one tile per workgroup stay below it.
constexpr uint32_t kMaxGrid = (1u << 24) - 1;

// Everything one kernel launch needs; passed by value in the kernel-argument
// segment, so no datatype metadata ever lives in device memory.
//
// The launch covers `nrows` runs of `n0` words of W bytes.  Row r is element
// (i_0, i_1, ...) of the row dimensions (r = i_0 + rcount[0]*(i_1 + ...)); its
// bytes sit at strided + sum(i_d * rstride[d]) and at packed + r * row_pitch.
//
// Words are "ragged": a run whose length is no multiple of W still moves in whole words, the
// last one pulled back by `tail_back` bytes so that it ends with the run and overlaps its
// neighbour (the overlap is written twice with the same bytes).  Neither side needs any
// alignment: the hardware takes unaligned vector accesses (the amdhsa ABI runs with
// SH_MEM_CONFIG.alignment_mode = unaligned, and the compiler is told so by the word types).
struct KParams {
    const char* strided = nullptr;  // typed buffer: origin + start (+ split offset)
    char* packed = nullptr;         // contiguous buffer + position (+ split offset)
    int64_t row_pitch = 0;          // bytes between consecutive rows in the packed stream
    uint32_t n0 = 0;                // words per run = ceil(run bytes / W)
    uint32_t nrows = 0;
    uint32_t bx_log2 = 0;           // lanes along a run = 1 << bx_log2; the other lanes take further rows
    uint32_t nxc = 1;               // x-chunks per row; block id = row_chunk * nxc + x_chunk
    uint32_t nrd = 0;               // row dimensions in use
    uint32_t tail_back = 0;         // n0 * W - run bytes (0 .. W-1): how far the last word is pulled back
    uint32_t ntiles = 0;            // tiles of the launch; workgroup g takes tiles g, g + gridDim.x, ...
    FastDiv xc_div;
    FastDiv rdiv[kMaxDims];
    uint32_t rcount[kMaxDims] = {};
    int64_t rstride[kMaxDims] = {};
};

// Parameters of the transposing kernel, for blocks whose elements (short runs of `ew` words of W
// bytes) are adjacent in the typed buffer along one row dimension ("A") while the packed stream
// runs along another ("B", the innermost row dimension): a plain row-by-row copy would touch one
// memory line per element on one side or the other.  Workgroups move te_a x te_b element tiles
// through LDS instead, reading along the dimension that is contiguous on the source side and
// writing along the one that is contiguous on the destination side.  This is where the stride
// order the paper's canonicalizer sorts by (Sec. 3.2, last pass) matters; the packed order itself
// stays the type-map order.
struct XParams {
    const char* strided = nullptr;  // typed buffer: origin + start
    char* packed = nullptr;         // contiguous buffer + position
    uint32_t ca = 0, cb = 0;        // element counts of the two tiled dimensions
    uint32_t ew = 1;                // words per element (element = ew << word_log2 bytes)
    uint32_t te_a = 0, te_b = 0;    // tile edges in elements (a thin dimension is covered whole, the other grows)
    uint32_t fa_log2 = 0, fb_log2 = 0;  // lanes along a tile row on the typed (A) and packed (B) side (rows of more words are walked in chunks)
    uint32_t pitch = 0;             // LDS row pitch in words (chosen so that column accesses spread over banks)
    int64_t tb_stride = 0;          // typed bytes between B-neighbours (A-neighbours are one element apart)
    int64_t pa_stride = 0;          // packed bytes between A-neighbours (B-neighbours are one element apart)
    uint32_t tiles_a = 0, tiles_b = 0;
    FastDiv tiles_a_div, tiles_b_div;
    uint32_t nod = 0;               // remaining ("outer") row dimensions, nesting order
    FastDiv odiv[kMaxDims];
    uint32_t ocount[kMaxDims] = {};
    int64_t otstride[kMaxDims] = {};  // typed bytes per step
    int64_t opstride[kMaxDims] = {};  // packed bytes per step
};

// Words along one row of a square tile of the transposing kernel, by word width: a tile row is
// 128 bytes to 1 KiB of contiguous memory.  The LDS tile holds xpose_lds_words() words (below 50 KiB).
constexpr int xpose_fast_words(int word_log2) { return word_log2 == 4 ? 32 : word_log2 >= 2 ? 64 : 128; }
// True if a launch has the shape the kernel's constant-parameter variant assumes.
inline bool xpose_is_square(const XParams& x, int word_log2) {
    const uint32_t edge = static_cast<uint32_t>(word_log2 == 4 ? 32 : word_log2 >= 2 ? 64 : 128);
    return x.ew == 1 && x.te_a == edge && x.te_b == edge && x.pitch == edge + 1;
}
constexpr int xpose_lds_words(int word_log2) { return xpose_fast_words(word_log2) * (xpose_fast_words(word_log2) + 32); }

// A pass that only reads (staged unpack, plan.cpp): the workgroup of tile t loads bytes
// [t * tile_bytes, (t + 1) * tile_bytes) of `base`, cut off at `bytes`, so that they sit in the L2 of
// the XCD that the same tile of the store passes behind it runs on.
struct PrefetchParams {
    const char* base = nullptr;
    uint64_t bytes = 0;       // at least 16
    uint32_t tile_bytes = 0;  // a power of two, at least 16
    uint32_t ntiles = 0;
};

enum LaunchKind : int { kTile = 0, kXpose = 1, kPrefetch = 2 };

struct Launch {
    KParams p;
    XParams x;          // kind == kXpose only
    PrefetchParams f;   // kind == kPrefetch only
    int kind = kTile;
    int word_log2 = 0;  // W = 1 << word_log2 bytes per lane access
    int ux = 1;         // words per thread along the run
    int ur = 1;         // rows per thread
    int nt = 3;         // streaming hints: bit 0 = non-temporal loads, bit 1 = non-temporal stores,
                        // bit 2 (with bit 1) = stores that L2 writes through at once
    uint32_t nblocks = 0;  // tiles
    uint32_t grid = 0;     // workgroups launched; 0 = one per tile
};

struct PlanInput {
    StridedBlock block;
    int64_t extent = 0;      // distance between consecutive objects
    int64_t count = 0;       // objects
    const char* typed = nullptr;   // origin of object 0 in the typed buffer
    char* packed = nullptr;        // contiguous buffer + position
    bool unpack = false;     // direction: the typed side is written
    bool packed_on_host = false;   // the contiguous buffer is mapped host memory (zero-copy)
    bool batched = false;          // one request of a batch call: small ones should stay fit for a batched launch
    bool narrow_partial_rows = true;  // override: unpack rows with partial memory lines in narrow words
    bool allow_xpose = true;          // override: permit the transposing kernel
    int max_word_log2 = 4;   // override: cap on the access width
    int nt = -1;             // override: streaming hints (-1 = planner's choice)
    int max_ur = -1;         // override: rows per thread in tiles for runs up to 256 words (-1 = planner's choice)
    int unpack_rule = 1;     // override: 0 = plan unpack launches as before write-through stores (for comparisons)
    int stage = -1;          // override: staged unpack of tiny rows: -1 = planner's choice, 0 = never, 1 = wherever it applies
    int64_t stage_bytes = int64_t{16} << 20;  // override: packed bytes per staged chunk
    int stage_grid = 0;      // override: workgroups of a staged launch (0 = planner's choice)
    int grid = 0;            // override: workgroups of every other row-by-row launch (0 = one per tile)
    int64_t max_rows_per_launch = int64_t{1} << 30;   // tests lower these to force splitting
    int64_t max_words_per_run = int64_t{1} << 30;
};

// Fills `out` (cleared first).  Returns a TP_* status.
int plan_launches(const PlanInput& in, std::vector<Launch>* out);

// ---- batched launches: many planned launches (of different datatypes) in one grid ----------
// The descriptors still travel in the kernel-argument segment (4 KiB at most), so each is
// packed into 96 bytes and limited to kBatchRowDims row dimensions.
constexpr int kBatchRowDims = 3;
constexpr int kBatchMax = 40;

struct BatchDesc {
    const char* strided;
    char* packed;
    int64_t row_pitch;
    int64_t rstride[kBatchRowDims];
    uint32_t rcount[kBatchRowDims];
    uint32_t rmul[kBatchRowDims];
    uint32_t n0, nrows, nxc, xc_mul;
    uint8_t rshift[kBatchRowDims];
    uint8_t xc_shift, bx_log2, word_log2;
    uint8_t tile;  // bits 0-1: 0 = (ux,ur) (1,4), 1 = (2,2), 2 = (4,1); bits 4-7: tail_back
    uint8_t nrd;   // 1..kBatchRowDims
};
static_assert(sizeof(BatchDesc) == 96, "BatchDesc must stay 96 bytes");

struct BatchParams {
    uint32_t n = 0;                    // descriptors in use
    uint32_t nblocks = 0;              // == block_end[n - 1]
    uint32_t block_end[kBatchMax] = {};  // descriptor j owns workgroups [block_end[j-1], block_end[j])
    BatchDesc d[kBatchMax];
};
static_assert(sizeof(BatchParams) <= 4096, "BatchParams must fit the kernel-argument segment");

// True if a launch can ride in a batch (few enough row dimensions).
bool batchable(const Launch& l);
// Groups launches into batches of at most kBatchMax descriptors, in order.  Launches that are
// not batchable are appended to `singles`.
void make_batches(const std::vector<Launch>& launches, std::vector<BatchParams>* batches,
                  std::vector<Launch>* singles);
std::string describe(const std::vector<BatchParams>& batches);

// One line per launch, for tp_last_plan().
std::string describe(const std::vector<Launch>& launches);

}  // namespace tp
