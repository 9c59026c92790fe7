#include "plan.hpp"

#include <algorithm>
#include <cstdio>

#include "status.hpp"

namespace tp {

namespace {

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
void choose_tile(uint32_t n0, Launch* l) {
    if (n0 >= 4u * kBlockThreads) {
        l->p.bx_log2 = 8;
        l->ux = 4;
        l->ur = 1;
    } else if (n0 > static_cast<uint32_t>(kBlockThreads)) {
        l->p.bx_log2 = 8;
        l->ux = n0 <= 2u * kBlockThreads ? 2 : 4;
        l->ur = 4 / l->ux;
    } else {
        l->p.bx_log2 = static_cast<uint32_t>(ceil_log2(n0));
        l->ux = 1;
        l->ur = 4;
    }
}

struct Splitter {
    const PlanInput& in;
    int kind;
    int word_log2;
    int64_t row_pitch;  // bytes of a full run in the packed stream
    std::vector<Launch>* out;

    // One launch over dims[0..nd): dims[0].count bytes per run (a multiple of the word).
    void add(const std::vector<Dim>& dims, const char* typed, char* packed) {
        Launch l;
        l.kind = kind;
        l.word_log2 = word_log2;
        KParams& p = l.p;
        p.strided = typed;
        p.packed = packed;
        p.row_pitch = row_pitch;
        p.run_len = static_cast<uint32_t>(dims[0].count);
        p.n0 = slots(dims[0].count);
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
        choose_tile(p.n0, &l);
        l.nt = in.nt >= 0 ? in.nt : 3;
        const uint32_t bx = 1u << p.bx_log2;
        const uint32_t br = kBlockThreads >> p.bx_log2;
        p.nxc = (p.n0 + bx * l.ux - 1) / (bx * l.ux);
        p.xc_div = make_fastdiv(p.nxc);
        const uint64_t nrc = (rows + uint64_t{br} * l.ur - 1) / (uint64_t{br} * l.ur);
        l.nblocks = static_cast<uint32_t>(nrc * p.nxc);
        out->push_back(l);
    }

    // Lane slots along a run of `bytes`: words, or for a shifted copy the whole 4-byte words of
    // the destination plus one slot for the ragged head and tail bytes.
    uint32_t slots(int64_t bytes) const {
        return static_cast<uint32_t>(kind == kShift ? (bytes >> word_log2) + 1 : bytes >> word_log2);
    }

    // Largest row count for which block ids stay below 2^30 with runs of n0 words.
    int64_t row_limit(int64_t n0) const {
        Launch probe;
        choose_tile(static_cast<uint32_t>(n0), &probe);
        const int64_t bx = int64_t{1} << probe.p.bx_log2;
        const int64_t br = kBlockThreads >> probe.p.bx_log2;
        const int64_t nxc = (n0 + bx * probe.ux - 1) / (bx * probe.ux);
        const int64_t by_blocks = ((int64_t{1} << 30) / nxc) * br * probe.ur;
        return std::max<int64_t>(1, std::min(in.max_rows_per_launch, by_blocks));
    }

    // Rows: split the outermost dimension until a launch's row count fits.
    void split_rows(std::vector<Dim> dims, const char* typed, char* packed) {
        int64_t rows = 1;
        for (size_t d = 1; d < dims.size(); ++d) rows *= dims[d].count;
        const int64_t limit = row_limit(slots(dims[0].count));
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

    // Runs longer than the per-launch word limit are cut into pieces along dimension 0.
    void split_runs(const std::vector<Dim>& dims, const char* typed, char* packed) {
        // a shifted-copy piece also has to keep its byte length in 32 bits
        const int64_t piece = kind == kShift ? std::min(in.max_words_per_run << word_log2, int64_t{1} << 30)
                                             : in.max_words_per_run << word_log2;
        for (int64_t off = 0; off < dims[0].count; off += piece) {
            std::vector<Dim> sub = dims;
            sub[0].count = std::min(piece, dims[0].count - off);
            split_rows(sub, typed + off, packed + off);
        }
    }
};

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

    // Word width: the widest power of two (at most 16 bytes) that divides the run length,
    // every stride and both start addresses, so that each access is naturally aligned.
    const char* typed = in.typed + sb.start;
    uint64_t bits = static_cast<uint64_t>(dims[0].count) | reinterpret_cast<uintptr_t>(typed) |
                    reinterpret_cast<uintptr_t>(in.packed);
    for (size_t d = 1; d < dims.size(); ++d)
        bits |= static_cast<uint64_t>(dims[d].stride < 0 ? -dims[d].stride : dims[d].stride);
    int word_log2 = std::min(4, in.max_word_log2);
    if (bits != 0) word_log2 = std::min(word_log2, __builtin_ctzll(bits));
    // Runs of at most 32 bytes: every run costs a whole 128-byte line whatever the word, and a
    // wavefront whose lanes share rows touches fewer lines per instruction.  Measured: gathers run
    // 5-13 % faster with four (or more) lanes per row than with one wide word per row, so cap the
    // word at a quarter of the run, and at 4 bytes.
    if (dims.size() > 1 && dims[0].count <= 32) {
        const int quarter_log2 = dims[0].count >= 4 ? 63 - __builtin_clzll(static_cast<uint64_t>(dims[0].count / 4)) : 0;
        word_log2 = std::min(word_log2, std::min(2, quarter_log2));
    }

    // Long runs that only byte- or 2-byte-wide words would fit move through the shifted copy.
    int kind = kTile;
    if (in.allow_shift && word_log2 < 2 && in.max_word_log2 >= 2 && dims[0].count >= 64) {
        kind = kShift;
        word_log2 = 2;
    }
    Splitter s{in, kind, word_log2, dims[0].count, out};
    s.split_runs(dims, typed, in.packed);
    return kSuccess;
}

bool batchable(const Launch& l) {
    return l.kind == kTile && l.p.nrd <= static_cast<uint32_t>(kBatchRowDims) && l.nblocks > 0;
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
    d.tile = static_cast<uint8_t>(l.ux == 1 ? 0 : l.ux == 2 ? 1 : 2);
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
        // block ids stay below 2^31 so the in-kernel multiply-shift division holds
        if (group.size() == static_cast<size_t>(kBatchMax) || group_blocks + l.nblocks >= (uint64_t{1} << 31)) flush();
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
        std::snprintf(line, sizeof line, "%s W=%d ux=%d ur=%d nt=%d bx=%u n0=%u rows=%u nrd=%u blocks=%u\n",
                      l.kind == kShift ? "shift" : "tile", 1 << l.word_log2, l.ux, l.ur, l.nt, 1u << l.p.bx_log2, l.p.n0, l.p.nrows, l.p.nrd, l.nblocks);
        text += line;
    }
    return text;
}

}  // namespace tp
