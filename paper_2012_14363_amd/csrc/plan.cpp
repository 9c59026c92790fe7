#include "plan.hpp"

#include <algorithm>
#include <limits>
#include <cstdio>

#include "status.hpp"

namespace tp {

namespace {

constexpr int64_t kPageBytes = 4096;  // rows at least this far apart each need their own address translation
constexpr int64_t kLineBytes = 128;   // memory line: what a partial write is read-modify-written in
constexpr int64_t kSoloRows = int64_t{1} << 20, kSoloBytes = int64_t{8} << 20;  // batch requests worth their own launch
constexpr int64_t kStagedRows = int64_t{1} << 19;  // fewer rows do not repay the extra passes (2^18: 15.0 against 14.5 us; 2^19: 22 against 26)
// Workgroups of a staged launch: a multiple of the eight XCDs.  Measured on 64 MiB of rows at 512-byte pitch, us for
// 96 / 128 / 160 / 192 / 224 / 256 / 320 workgroups: 1-byte rows 1766 / 1779 / 1777 / 1750 / 1779 / 1784 / 2097, 2-byte rows
// 894 / 902 / 892 / 882 / 906 / 971 / -, 8-byte rows 244 / 249 / 243 / 241 / 246 / 259 / -: a flat optimum from 168 to 208.
constexpr uint32_t kStagedGrid = 192;
constexpr uint32_t kPrefetchGridFactor = 8;        // the read-only pass takes that many times more

struct Dim {
    int64_t count;
    int64_t stride;
};

int ceil_log2(uint64_t v) {
    int s = 0;
    while ((uint64_t{1} << s) < v) ++s;
    return s;
}

// Thread-tile shape for runs of n0 words (Sec. 3.3 maps X to the run and fills the
// block with further rows; here the block is flat and the split is a power of two).
// Runs longer than the workgroup are cut into chunks of 256 * ux words; of ux = 1, 2, 4 the one
// that pads the run least wins (1025 words: five chunks of 256 rather than two of 1024), the
// larger on a tie since its row arithmetic is scalar.
// `ur_short`: rows per thread (1 or 4) where a run fits the workgroup.
void choose_tile(uint32_t n0, int ur_short, Launch* l) {
    if (n0 <= static_cast<uint32_t>(kBlockThreads)) {
        l->p.bx_log2 = static_cast<uint32_t>(ceil_log2(n0));
        l->ux = 1;
        l->ur = ur_short;
        return;
    }
    l->p.bx_log2 = 8;
    uint64_t best = ~uint64_t{0};
    for (int ux : {4, 2, 1}) {
        const uint64_t chunk = static_cast<uint64_t>(kBlockThreads) * ux;
        const uint64_t padded = (n0 + chunk - 1) / chunk * chunk;
        if (padded < best) {
            best = padded;
            l->ux = ux;
        }
    }
    l->ur = 4 / l->ux;
}

struct Splitter {
    const PlanInput& in;
    int word_log2;
    int64_t row_pitch;  // bytes of a full run in the packed stream
    std::vector<Launch>* out;
    int ur_short = 4;   // rows per thread in tiles for runs that fit the workgroup
    int nt = 3;         // streaming hints of the launches
    uint32_t grid = 0;  // workgroups per launch (0 = one per tile)
    int64_t chunk_rows = 0;  // > 0: no launch of more rows (staged unpack)

    int64_t word() const { return int64_t{1} << word_log2; }
    // Words that cover a run of `bytes` (>= one word): the last one may overlap its neighbour.
    uint32_t words(int64_t bytes) const { return static_cast<uint32_t>((bytes + word() - 1) >> word_log2); }

    // One launch over dims[0..nd): dims[0].count bytes per run.
    void add(const std::vector<Dim>& dims, const char* typed, char* packed) {
        Launch l;
        l.word_log2 = word_log2;
        KParams& p = l.p;
        p.strided = typed;
        p.packed = packed;
        p.row_pitch = row_pitch;
        p.n0 = words(dims[0].count);
        p.tail_back = static_cast<uint32_t>((static_cast<int64_t>(p.n0) << word_log2) - dims[0].count);
        uint64_t rows = 1;
        p.nrd = 0;
        for (size_t d = 1; d < dims.size(); ++d) {
            if (dims[d].count == 1) continue;
            p.rcount[p.nrd] = static_cast<uint32_t>(dims[d].count);
            p.rstride[p.nrd] = dims[d].stride;
            p.rdiv[p.nrd] = make_fastdiv(p.rcount[p.nrd]);
            ++p.nrd;
            rows *= static_cast<uint64_t>(dims[d].count);
        }
        p.nrows = static_cast<uint32_t>(rows);
        choose_tile(p.n0, ur_short, &l);
        l.nt = nt;
        const uint32_t bx = 1u << p.bx_log2;
        const uint32_t br = kBlockThreads >> p.bx_log2;
        p.nxc = (p.n0 + bx * l.ux - 1) / (bx * l.ux);
        p.xc_div = make_fastdiv(p.nxc);
        const uint64_t nrc = (rows + uint64_t{br} * l.ur - 1) / (uint64_t{br} * l.ur);
        l.nblocks = static_cast<uint32_t>(nrc * p.nxc);
        if (grid) l.grid = std::min(grid, l.nblocks);
        else if (l.nblocks > kMaxGrid) l.grid = kMaxGrid;   // more tiles than a grid may have workgroups
        out->push_back(l);
    }

    // Largest row count for which block ids stay below 2^30 with runs of n0 words.
    int64_t row_limit(int64_t n0) const {
        Launch probe;
        choose_tile(static_cast<uint32_t>(n0), ur_short, &probe);
        const int64_t bx = int64_t{1} << probe.p.bx_log2;
        const int64_t br = kBlockThreads >> probe.p.bx_log2;
        const int64_t nxc = (n0 + bx * probe.ux - 1) / (bx * probe.ux);
        const int64_t by_blocks = ((int64_t{1} << 30) / nxc) * br * probe.ur;
        const int64_t limit = std::min(in.max_rows_per_launch, by_blocks);
        return std::max<int64_t>(1, chunk_rows > 0 ? std::min(limit, chunk_rows) : limit);
    }

    // Rows: split the outermost dimension until a launch's row count fits.
    void split_rows(std::vector<Dim> dims, const char* typed, char* packed) {
        int64_t rows = 1;
        for (size_t d = 1; d < dims.size(); ++d) rows *= dims[d].count;
        const int64_t limit = row_limit(words(dims[0].count));
        if (rows <= limit) {
            add(dims, typed, packed);
            return;
        }
        const Dim top = dims.back();
        const int64_t inner_rows = rows / top.count;
        const int64_t chunk = std::max<int64_t>(1, limit / inner_rows);
        for (int64_t i = 0; i < top.count; i += chunk) {
            const int64_t k = std::min(chunk, top.count - i);
            std::vector<Dim> sub = dims;
            if (inner_rows > limit) sub.pop_back(); else sub.back().count = k;
            split_rows(sub, typed + i * top.stride, packed + i * inner_rows * row_pitch);
        }
    }

    // Runs longer than the per-launch word limit are cut into pieces along dimension 0.  A piece
    // is a run of its own and needs at least one word, so a last piece shorter than that starts
    // early instead and overlaps the piece before it (same bytes written twice).
    void split_runs(const std::vector<Dim>& dims, const char* typed, char* packed) {
        const int64_t piece = in.max_words_per_run << word_log2;
        const int64_t total = dims[0].count;
        for (int64_t off = 0; off < total; off += piece) {
            int64_t at = off, len = std::min(piece, total - off);
            if (len < word()) {
                at = total - word();
                len = word();
            }
            std::vector<Dim> sub = dims;
            sub[0].count = len;
            split_rows(sub, typed + at, packed + at);
        }
    }
};

// The transposing kernel (plan.hpp: XParams) applies when the elements are short runs (a few
// words of the widest power of two dividing their length) and some outer row dimension A steps
// by exactly one element while the innermost row dimension B strides over at least two.  Returns false (and leaves `out` alone) when it does not apply or the launch would not
// fit one grid.
bool plan_xpose(const PlanInput& in, const std::vector<Dim>& dims, const char* typed, std::vector<Launch>* out) {
    if (!in.allow_xpose || dims.size() < 3) return false;
    const int64_t run = dims[0].count;
    if (run > 64) return false;
    const int word_log2 = std::min({4, in.max_word_log2, __builtin_ctzll(static_cast<uint64_t>(run))});
    const int64_t ew = run >> word_log2;
    // Edge of a square tile, in elements: one-word elements use the power of two the kernel's
    // constant-parameter variant is built for; elements of several words take the largest edge
    // whose rows fit the workgroup (256 words) and whose tile fits LDS.
    const int64_t lds_words = xpose_lds_words(word_log2);
    int64_t square = xpose_fast_words(word_log2);
    if (ew > 1) {
        square = kBlockThreads / ew;
        while (square > 0 && square * (square * ew + 32) > lds_words) --square;
    }
    if (square < 12) return false;
    // tests that lower the split limits mean the row-by-row kernel
    if (in.max_rows_per_launch != (int64_t{1} << 30) || in.max_words_per_run != (int64_t{1} << 30)) return false;
    const Dim& b = dims[1];
    size_t a = 0;
    for (size_t d = 2; d < dims.size() && a == 0; ++d)
        if (dims[d].stride == run && dims[d].count >= 2) a = d;
    if (a == 0) return false;
    // A dimension of very few elements (records of two or three fields): the row-by-row kernel's
    // re-reads mostly hit in cache, and tiles that thin give a workgroup little to do.  Measured on
    // 4 Mi records of 8-byte fields, row by row against transposing, pack / unpack in us: three fields
    // 72 / 120 against 84 / 87, four fields 110 / 224 against 86 / 89, eight 376 / 876 against 108 / 111.
    const int64_t thin = std::min(dims[a].count, b.count);
    if (thin < (in.unpack ? 3 : 4)) return false;
    // Walking B row by row uses one element of every |stride| bytes and comes back for the rest
    // on later rows: worth transposing from an amplification of two, given enough elements.
    const int64_t bstep = b.stride < 0 ? -b.stride : b.stride;
    if (bstep < 2 * run || dims[a].count * b.count < 1024) return false;

    // Tile shape: square where both dimensions are long; a dimension shorter than half an edge is
    // covered whole and the other edge grows (as far as LDS reaches), so that a workgroup still
    // has tens of KiB to move.
    int64_t te_a = std::min<int64_t>(square, dims[a].count), te_b = std::min<int64_t>(square, b.count);
    // LDS row pitch in words: at least a tile row, and such that lanes walking down a tile
    // column fall into distinct banks (32 of them): any odd pitch for one-word elements, a pitch
    // congruent to ew modulo 32 for elements of ew words.
    auto pitch_for = [ew](int64_t edge_a) {
        uint32_t pitch = static_cast<uint32_t>(edge_a * ew);
        if (ew == 1) return pitch | 1u;
        while (pitch % 32 != static_cast<uint32_t>(ew % 32)) ++pitch;
        return pitch;
    };
    uint32_t pitch = pitch_for(te_a);
    constexpr int64_t kLongEdge = 1024;  // elements along the grown edge of a thin tile, at most
    // a grown edge beyond one chunk of lanes is a whole number of chunks
    auto whole_chunks = [ew](int64_t edge) {
        const int64_t chunk = kBlockThreads / ew;
        return edge > chunk ? edge / chunk * chunk : edge;
    };
    if (te_a * 2 <= square) te_b = whole_chunks(std::min({b.count, kLongEdge, lds_words / pitch}));
    else if (te_b * 2 <= square) {
        te_a = whole_chunks(std::min({dims[a].count, kLongEdge, (lds_words / te_b - 32) / ew}));
        if (te_a < 1) return false;
        pitch = pitch_for(te_a);
    }
    if (te_b * pitch > lds_words) return false;

    Launch l;
    l.kind = kXpose;
    l.word_log2 = word_log2;
    l.nt = 3;
    XParams& x = l.x;
    x.strided = typed;
    x.packed = in.packed;
    x.ca = static_cast<uint32_t>(dims[a].count);
    x.cb = static_cast<uint32_t>(b.count);
    x.ew = static_cast<uint32_t>(ew);
    x.te_a = static_cast<uint32_t>(te_a);
    x.te_b = static_cast<uint32_t>(te_b);
    x.fa_log2 = static_cast<uint32_t>(std::min(8, ceil_log2(static_cast<uint64_t>(te_a * ew))));
    x.fb_log2 = static_cast<uint32_t>(std::min(8, ceil_log2(static_cast<uint64_t>(te_b * ew))));
    x.pitch = pitch;
    x.tb_stride = b.stride;
    x.tiles_a = static_cast<uint32_t>((dims[a].count + te_a - 1) / te_a);
    x.tiles_b = static_cast<uint32_t>((b.count + te_b - 1) / te_b);
    x.tiles_a_div = make_fastdiv(x.tiles_a);
    x.tiles_b_div = make_fastdiv(x.tiles_b);
    // packed bytes per step of row dimension d: one element times the counts nested inside it
    int64_t pstride = run;
    uint64_t blocks = static_cast<uint64_t>(x.tiles_a) * x.tiles_b;
    for (size_t d = 1; d < dims.size(); ++d) {
        if (d == a) {
            x.pa_stride = pstride;
        } else if (d != 1 && dims[d].count != 1) {
            x.ocount[x.nod] = static_cast<uint32_t>(dims[d].count);
            x.odiv[x.nod] = make_fastdiv(x.ocount[x.nod]);
            x.otstride[x.nod] = dims[d].stride;
            x.opstride[x.nod] = pstride;
            ++x.nod;
            blocks *= static_cast<uint64_t>(dims[d].count);
            if (blocks > kMaxGrid) return false;
        }
        pstride *= dims[d].count;
    }
    if (blocks > kMaxGrid) return false;   // one tile per workgroup
    l.nblocks = static_cast<uint32_t>(blocks);
    out->push_back(l);
    return true;
}

// Staged unpack of tiny rows.  Partially written memory lines retire about 1.5 times faster when
// (a) the lines written at one time are exactly 512 bytes apart and (b) no read from HBM falls
// between the writes (measured with one-byte rows: 37 G rows/s against 19 to 25 G at any other
// spacing from 64 to 4096 bytes, and against 22 G with the source streamed from HBM; 64 MiB of
// one-byte rows at 512-byte pitch unpack in 1.8 ms instead of 2.7).  For rows of one word each at a
// pitch of 512 bytes, or of 256 or 128 taken in 2 or 4 passes over every 2nd or 4th row, the
// launch is therefore cut into chunks of `stage_bytes` packed bytes, and every chunk becomes a
// read-only pass that brings its packed bytes into L2 followed by the store passes, all with the
// same few workgroups taking the same tiles: workgroup ids map to XCDs round-robin, so a tile's
// bytes wait in the L2 its stores will ask.  Returns false where this does not apply.
bool plan_staged(const PlanInput& in, const std::vector<Dim>& all_dims, const char* typed, std::vector<Launch>* out) {
    std::vector<Dim> dims = {all_dims[0]};
    for (size_t d = 1; d < all_dims.size(); ++d)
        if (all_dims[d].count != 1) dims.push_back(all_dims[d]);   // a dimension of one row is none
    if (dims.size() < 2) return false;
    const int64_t run = dims[0].count, pitch = dims[1].stride;
    int64_t rows = 1;
    for (size_t d = 1; d < dims.size(); ++d) rows *= dims[d].count;
    const int64_t step = pitch < 0 ? -pitch : pitch;
    if (run > 16 || (run & (run - 1)) != 0 || (int64_t{1} << in.max_word_log2) < run) return false;
    if (step != 128 && step != 256 && step != 512) return false;
    if (dims.size() > 2 && step != 512) return false;   // passes over every 2nd or 4th row: one row dimension only
    // rows in the last of the four lines of their 512-byte block do not reach the fast rate (measured: a
    // column of 8-byte elements at byte 384 or beyond of 512-byte matrix rows unpacks as without staging)
    if (step == 512 && in.stage != 1 && (reinterpret_cast<uintptr_t>(typed) & 511u) >= 384u) return false;
    if (in.stage != 1 && rows < kStagedRows) return false;
    if (in.max_rows_per_launch != (int64_t{1} << 30) || in.max_words_per_run != (int64_t{1} << 30)) return false;
    const int64_t passes = 512 / step;
    // the passes give up the locality of neighbouring rows, which costs more the more of each line the
    // rows fill: measured to pay for 1- to 16-byte rows at 512-byte pitch, up to 4 bytes at 256, 1 byte at 128
    if (run * passes * passes > 16) return false;
    const int64_t tile_rows = int64_t{kBlockThreads} * passes;  // rows of all passes that share one tile index
    // tile_rows * run bytes per tile: a power of two, at least 256
    int64_t chunk_rows = std::max<int64_t>(in.stage_bytes / run, 1) / tile_rows * tile_rows;
    if (chunk_rows == 0) chunk_rows = tile_rows;
    const uint32_t grid = in.stage_grid > 0 ? static_cast<uint32_t>(in.stage_grid) : kStagedGrid;
    int word_log2 = 0;
    while ((int64_t{1} << word_log2) < run) ++word_log2;
    auto add_prefetch = [&](const char* base, int64_t nrows) {
        if (nrows * run < 16) return;   // the read-only pass loads 16-byte words
        Launch l;
        l.kind = kPrefetch;
        l.f.base = base;
        l.f.bytes = static_cast<uint64_t>(nrows * run);
        l.f.tile_bytes = static_cast<uint32_t>(tile_rows * run);
        l.f.ntiles = static_cast<uint32_t>((nrows + tile_rows - 1) / tile_rows);
        l.nblocks = l.f.ntiles;
        // more workgroups than the store passes have (the read is over sooner), still a multiple of the
        // eight XCDs, so tile t lands on XCD t mod 8 here as there
        l.grid = std::min(grid * kPrefetchGridFactor, l.nblocks);
        out->push_back(l);
    };
    if (dims.size() > 2) {
        // several row dimensions (512-byte pitch, one pass): the splitter cuts the outer dimensions into
        // launches of at most a chunk's rows, consecutive in the packed stream; each gets its pass in front
        std::vector<Launch> cut;
        Splitter s{in, word_log2, run, &cut, 1, in.nt >= 0 ? in.nt : 6, grid, chunk_rows};
        s.split_rows(dims, typed, in.packed);
        for (const Launch& l : cut) {
            add_prefetch(l.p.packed, static_cast<int64_t>(l.p.nrows));
            out->push_back(l);
        }
        return true;
    }
    for (int64_t lo = 0; lo < rows; lo += chunk_rows) {
        const int64_t n = std::min(chunk_rows, rows - lo);
        add_prefetch(in.packed + lo * run, n);
        for (int64_t p = 0; p < passes && p < n; ++p) {
            // rows lo + p, lo + p + passes, ...: `passes` rows apart on both sides
            Splitter s{in, word_log2, run * passes, out, 1, in.nt >= 0 ? in.nt : 6, grid};
            const std::vector<Dim> sub = {{run, 1}, {(n - p + passes - 1) / passes, pitch * passes}};
            s.add(sub, typed + (lo + p) * pitch, in.packed + (lo + p) * run);
        }
    }
    return true;
}

}  // namespace

int plan_launches(const PlanInput& in, std::vector<Launch>* out) {
    out->clear();
    const StridedBlock& sb = in.block;
    if (in.count == 0 || sb.counts[0] == 0) return kSuccess;

    std::vector<Dim> dims;
    for (int d = 0; d < sb.ndims; ++d) dims.push_back({sb.counts[d], sb.strides[d]});
    // The object count is one more outer dimension of stride `extent` (Sec. 3.3 handles it
    // with the grid's Z dimension); fold or flatten it away when objects abut.
    if (in.count > 1) {
        Dim& top = dims.back();
        const int64_t top_span = dims.size() == 1 ? top.count : top.count * top.stride;
        if (in.extent == top_span) top.count *= in.count;
        else dims.push_back({in.count, in.extent});
    }
    if (dims.size() - 1 > static_cast<size_t>(kMaxDims)) return kErrRange;

    // Word width.  Words may sit at any address and need not divide the run (KParams: ragged
    // words, unaligned accesses), so the choice is free of both; measurements decide it.
    // Reading the typed side (pack): 16 bytes wherever a run holds that much - equal to narrower
    // words on runs they divide, up to 20 % faster on the others, and 2-4 times faster than the
    // bytes that natural alignment would force at odd addresses or run lengths.
    // Writing the typed side (unpack): a row that is not made of whole aligned 128-byte lines ends
    // in partially written lines, which the memory system read-modify-writes, and how the row's
    // stores are issued then matters: see the write-through rule below.  Where that rule does not
    // apply, the earlier one holds.  It was measured with plain streaming stores and four rows per
    // thread on 60 MiB of rows at 128- to 8192-byte pitch (4 / 8 / 16-byte words, us): 100-byte rows
    // 34 / 44 / 49, 200: 33 / 40 / 40, 1000: 29 / 33 / 35, but 1040: 34 / 27 / 27, 2056: 30 / 27 / 32,
    // 4100: 27 / 26 / 25: 4-byte words up to 1 KiB and 8-byte words beyond.  Rows of whole aligned
    // lines keep 16.
    const char* typed = in.typed + sb.start;
    if (plan_xpose(in, dims, typed, out)) return kSuccess;
    const int64_t run = dims[0].count;
    int word_log2 = std::min({4, in.max_word_log2, 63 - __builtin_clzll(static_cast<uint64_t>(run))});
    int ur_short = 4, nt = 3;
    // Do the typed rows consist of whole aligned 128-byte memory lines?  How far apart are rows that follow
    // one another in the packed stream (the innermost row dimension), and how close do rows come
    // that are written far apart in time (the outer row dimensions)?
    bool partial_rows = false;
    int64_t inner_pitch = 0, outer_pitch = std::numeric_limits<int64_t>::max();
    if (dims.size() > 1) {
        uint64_t bits = static_cast<uint64_t>(run) | reinterpret_cast<uintptr_t>(typed);
        for (size_t d = 1; d < dims.size(); ++d) {
            const int64_t step = dims[d].stride < 0 ? -dims[d].stride : dims[d].stride;
            bits |= static_cast<uint64_t>(step);
            if (dims[d].count == 1) continue;
            if (inner_pitch == 0) inner_pitch = step;
            else outer_pitch = std::min(outer_pitch, step);
        }
        partial_rows = (bits & static_cast<uint64_t>(kLineBytes - 1)) != 0;
    }
    // A request of a batch call keeps a plan the batched kernel can run unless it is large enough
    // for a launch of its own to pay (a launch costs about 5 us on the stream).
    int64_t rows = 1;
    for (size_t d = 1; d < dims.size(); ++d) rows *= dims[d].count;
    const bool own_launch = !in.batched || rows >= kSoloRows || rows * run >= kSoloBytes;
    if (in.unpack && !in.packed_on_host && in.unpack_rule == 1 && in.narrow_partial_rows && partial_rows &&
        inner_pitch < kPageBytes && outer_pitch >= kLineBytes && own_launch) {
        if (in.stage != 0 && plan_staged(in, dims, typed, out)) return kSuccess;
        // Rows that end in partially written memory lines, follow one another closer than a page and
        // share no line with rows of another outer index (those L2 should keep and merge): their
        // stores are written through L2 at once (`sc1 nt`) rather than left for eviction, a thread
        // takes one row, not four, and a row is spread over 8 to 15 lanes.  Measured on 32 MiB of rows
        // from rotating sources, against four rows per thread and plain streaming stores in 4-byte
        // words, us: 512-byte pitch: 12-byte rows 130 -> 112, 48: 39 -> 32, 100: 31 -> 23, 200: 20.4 ->
        // 18.7; 128-byte pitch: 16-byte rows 95 -> 57; 64-byte rows (half lines) at 256: 36 -> 29.  Rows
        // a page or more apart lose a few per cent this way (each row its own address translation,
        // which four rows per thread hide better), whole-line rows gain nothing.
        nt = 7;
        ur_short = 1;
        const int eighth_log2 = run >= 16 ? 63 - __builtin_clzll(static_cast<uint64_t>(run / 8)) : 0;
        word_log2 = std::min(word_log2, eighth_log2);
    } else {
        if (in.unpack && in.narrow_partial_rows && partial_rows) word_log2 = std::min(word_log2, run <= 1024 ? 2 : 3);
        // Reading mapped host memory across PCIe (zero-copy unpack): 16-byte loads were measured
        // slower than 8- or 4-byte ones (4 MiB: 115 us against 87; 64 MiB: 1270 against 1180), writes
        // to it do not care.
        if (in.unpack && in.packed_on_host) word_log2 = std::min(word_log2, 3);
        // Runs of at most 32 bytes: every run costs a whole 128-byte line whatever the word, and a
        // wavefront whose lanes share rows touches fewer lines per instruction.  Measured: gathers run
        // 5-13 % faster with four (or more) lanes per row than with one wide word per row, so cap the
        // word at a quarter of the run, and at 4 bytes.
        if (dims.size() > 1 && run <= 32) {
            const int quarter_log2 = run >= 4 ? 63 - __builtin_clzll(static_cast<uint64_t>(run / 4)) : 0;
            word_log2 = std::min(word_log2, std::min(2, quarter_log2));
        }
    }
    if (in.nt >= 0) nt = in.nt;
    if (in.max_ur == 1 || in.max_ur == 4) ur_short = in.max_ur;
    Splitter s{in, word_log2, run, out, ur_short, nt, in.grid > 0 ? static_cast<uint32_t>(in.grid) : 0u};
    s.split_runs(dims, typed, in.packed);
    return kSuccess;
}

bool batchable(const Launch& l) {
    // the batched kernel carries the three four-words-per-thread tiles and plain streaming hints
    return l.kind == kTile && l.p.nrd <= static_cast<uint32_t>(kBatchRowDims) && l.nblocks > 0 && l.ux * l.ur == 4 &&
           (l.nt & 4) == 0 && l.grid == 0;
}

namespace {

BatchDesc make_desc(const Launch& l) {
    BatchDesc d;
    const KParams& p = l.p;
    d.strided = p.strided;
    d.packed = p.packed;
    d.row_pitch = p.row_pitch;
    d.n0 = p.n0;
    d.nrows = p.nrows;
    d.nxc = p.nxc;
    d.xc_mul = p.xc_div.mul;
    d.xc_shift = static_cast<uint8_t>(p.xc_div.shift);
    d.bx_log2 = static_cast<uint8_t>(p.bx_log2);
    d.word_log2 = static_cast<uint8_t>(l.word_log2);
    d.tile = static_cast<uint8_t>((l.ux == 1 ? 0 : l.ux == 2 ? 1 : 2) | (p.tail_back << 4));
    d.nrd = static_cast<uint8_t>(p.nrd == 0 ? 1 : p.nrd);
    const FastDiv one = make_fastdiv(1);
    for (int k = 0; k < kBatchRowDims; ++k) {
        const bool used = static_cast<uint32_t>(k) < p.nrd;
        d.rstride[k] = used ? p.rstride[k] : 0;
        d.rcount[k] = used ? p.rcount[k] : 1;
        d.rmul[k] = used ? p.rdiv[k].mul : one.mul;
        d.rshift[k] = static_cast<uint8_t>(used ? p.rdiv[k].shift : one.shift);
    }
    return d;
}

}  // namespace

void make_batches(const std::vector<Launch>& launches, std::vector<BatchParams>* batches,
                  std::vector<Launch>* singles) {
    std::vector<const Launch*> group;
    uint64_t group_blocks = 0;
    auto flush = [&] {
        if (group.empty()) return;
        // Largest first: workgroups are handed out in index order, so the big descriptors start
        // while the whole chip is free and the small ones fill in behind them.  Each descriptor
        // carries its own addresses, so the order inside a launch is free.
        std::stable_sort(group.begin(), group.end(),
                         [](const Launch* a, const Launch* b) { return a->nblocks > b->nblocks; });
        BatchParams cur;
        for (const Launch* l : group) {
            cur.d[cur.n] = make_desc(*l);
            cur.nblocks += l->nblocks;
            cur.block_end[cur.n] = cur.nblocks;
            ++cur.n;
        }
        batches->push_back(cur);
        group.clear();
        group_blocks = 0;
    };
    for (const Launch& l : launches) {
        if (!batchable(l)) {
            singles->push_back(l);
            continue;
        }
        // one tile per workgroup: a batch has at most as many tiles as a grid may have workgroups
        if (group.size() == static_cast<size_t>(kBatchMax) || group_blocks + l.nblocks > kMaxGrid) flush();
        group.push_back(&l);
        group_blocks += l.nblocks;
    }
    flush();
}

std::string describe(const std::vector<BatchParams>& batches) {
    std::string text;
    char line[128];
    for (const BatchParams& b : batches) {
        std::snprintf(line, sizeof line, "batch descriptors=%u blocks=%u\n", b.n, b.nblocks);
        text += line;
    }
    return text;
}

std::string describe(const std::vector<Launch>& launches) {
    std::string text;
    char line[256];
    for (const Launch& l : launches) {
        if (l.kind == kXpose) {
            std::snprintf(line, sizeof line, "xpose W=%d words=%u tile=%ux%u a=%u b=%u outer=%u blocks=%u\n", 1 << l.word_log2,
                          l.x.ew, l.x.te_a, l.x.te_b, l.x.ca, l.x.cb, l.x.nod, l.nblocks);
            text += line;
            continue;
        }
        if (l.kind == kPrefetch) {
            std::snprintf(line, sizeof line, "prefetch bytes=%llu tile=%u blocks=%u grid=%u\n",
                          static_cast<unsigned long long>(l.f.bytes), l.f.tile_bytes, l.nblocks, l.grid ? l.grid : l.nblocks);
            text += line;
            continue;
        }
        std::snprintf(line, sizeof line, "tile W=%d ux=%d ur=%d nt=%d bx=%u n0=%u back=%u rows=%u nrd=%u blocks=%u",
                      1 << l.word_log2, l.ux, l.ur, l.nt, 1u << l.p.bx_log2, l.p.n0, l.p.tail_back, l.p.nrows, l.p.nrd, l.nblocks);
        text += line;
        if (l.grid) {
            std::snprintf(line, sizeof line, " grid=%u", l.grid);
            text += line;
        }
        text += "\n";
    }
    return text;
}

}  // namespace tp
