#include "canon.hpp"

#include "status.hpp"

namespace tp {

// ------------------------------------------------------------------ Sec. 3.1
static void translate_into(const TypeNode& t, Chain& chain) {
    switch (t.kind) {
    case Kind::Named: {
        // from_named: a DenseData as long as the named type, offset 0.
        Level d;
        d.dense = true;
        d.extent = t.size;
        chain.push_back(d);
        return;
    }
    case Kind::Contiguous: {
        // from_contiguous: a stream whose stride is the oldtype's extent (not a
        // DenseData: the oldtype may have holes).
        Level s;
        s.stride = t.old->extent();
        s.count = t.count;
        chain.push_back(s);
        break;
    }
    case Kind::Vector:
    case Kind::Hvector: {
        // from_vector / from_hvector: parent stream = the blocks, child stream =
        // the elements of one block.
        Level parent, child;
        child.stride = t.old->extent();
        child.count = t.blocklength;
        parent.stride = t.kind == Kind::Vector ? t.stride * child.stride : t.stride;
        parent.count = t.count;
        chain.push_back(parent);
        chain.push_back(child);
        break;
    }
    case Kind::Subarray: {
        // from_subarray: one stream per dimension.  The slowest-varying dimension
        // is the outermost stream: dimension 0 in C order, the last in Fortran
        // order.  stride_d = extent(old) * product of the sizes of all
        // faster-varying dimensions; offset_d = start_d * stride_d.
        const int n = static_cast<int>(t.sizes.size());
        int64_t pitch[kMaxDims];
        int64_t run = t.old->extent();
        for (int k = 0; k < n; ++k) {
            const int d = t.order == 0 ? n - 1 - k : k;  // fastest dimension first
            pitch[d] = run;
            run *= t.sizes[d];
        }
        for (int k = 0; k < n; ++k) {
            const int d = t.order == 0 ? k : n - 1 - k;  // slowest dimension first
            Level s;
            s.stride = pitch[d];
            s.count = t.subsizes[d];
            s.offset = t.starts[d] * pitch[d];
            chain.push_back(s);
        }
        break;
    }
    }
    translate_into(*t.old, chain);
}

Chain translate(const TypeNode& type) {
    Chain chain;
    chain.reserve(2 * kMaxDims);  // one allocation for all but the deepest trees
    translate_into(type, chain);
    return chain;
}

// ------------------------------------------------------------------ Sec. 3.2
// Alg. 2: a stream whose stride equals the extent of the DenseData below it is
// one longer DenseData.  Only the bottom pair can ever match, so fold upward
// from the leaf for as long as it does.
bool dense_folding(Chain& chain) {
    bool changed = false;
    while (chain.size() >= 2) {
        Level& leaf = chain.back();
        const Level& parent = chain[chain.size() - 2];
        if (!leaf.dense || parent.dense || parent.stride != leaf.extent) break;
        Level folded;
        folded.dense = true;
        folded.offset = leaf.offset + parent.offset;
        folded.extent = parent.count * parent.stride;
        chain.pop_back();
        chain.back() = folded;
        changed = true;
    }
    return changed;
}

// Alg. 3, read as: a stream of one element is that element, wherever it sits in
// the chain (root included); its offset moves to the level below it.
bool stream_elision(Chain& chain) {
    bool changed = false;
    for (size_t i = 0; i + 1 < chain.size();) {
        if (!chain[i].dense && chain[i].count == 1) {
            chain[i + 1].offset += chain[i].offset;
            chain.erase(chain.begin() + static_cast<long>(i));
            changed = true;
        } else {
            ++i;
        }
    }
    return changed;
}

// Alg. 4: when the parent's stride equals count x stride of the child stream,
// parent element p, child element c sits at (p * child.count + c) * child.stride:
// one stream.  Bottom-up, as in the listing.
bool stream_flatten(Chain& chain) {
    bool changed = false;
    for (size_t i = chain.size(); i-- > 1;) {
        Level& parent = chain[i - 1];
        const Level& child = chain[i];
        if (parent.dense || child.dense) continue;
        if (parent.stride != child.count * child.stride) continue;
        parent.count *= child.count;
        parent.stride = child.stride;
        parent.offset += child.offset;
        chain.erase(chain.begin() + static_cast<long>(i));
        changed = true;
    }
    return changed;
}

// Alg. 1: repeat the passes until none changes the chain.  The paper's fourth
// pass, sorting streams by stride, is left out on purpose: it would reorder
// dimensions and with them the order bytes appear in the packed stream, which
// MPI fixes as the type-map order.
void simplify(Chain& chain) {
    bool changed = true;
    while (changed) {
        changed = false;
        changed |= dense_folding(chain);
        changed |= stream_elision(chain);
        changed |= stream_flatten(chain);
    }
}

// ------------------------------------------------------------------ Sec. 3.3
// Alg. 5, walking from the DenseData leaf (dimension 0, stride 1) up to the root.
int strided_block(const Chain& chain, StridedBlock* out) {
    if (chain.empty() || !chain.back().dense) return kErrType;
    if (chain.size() > static_cast<size_t>(kMaxDims)) return kErrRange;
    StridedBlock sb;
    const Level& leaf = chain.back();
    sb.start = leaf.offset;
    sb.counts[0] = leaf.extent;
    sb.strides[0] = 1;
    sb.ndims = 1;
    for (size_t i = chain.size() - 1; i-- > 0;) {
        const Level& s = chain[i];
        if (s.dense) return kErrType;  // not strided
        sb.start += s.offset;
        sb.counts[sb.ndims] = s.count;
        sb.strides[sb.ndims] = s.stride;
        ++sb.ndims;
    }
    *out = sb;
    return kSuccess;
}

int canonicalize(const TypeNode& type, StridedBlock* out) {
    if (type.size == 0) {
        StridedBlock sb;
        sb.ndims = 1;
        sb.counts[0] = 0;
        sb.strides[0] = 1;
        *out = sb;
        return kSuccess;
    }
    Chain chain = translate(type);
    simplify(chain);
    return strided_block(chain, out);
}

int commit(const TypeNode& node) {
    std::call_once(node.commit_once, [&node] {
        StridedBlock sb;
        const int rc = canonicalize(node, &sb);
        node.commit_status = rc;
        if (rc != kSuccess) return;
        node.block = sb;
        node.committed.store(true, std::memory_order_release);
    });
    return node.commit_status;
}

}  // namespace tp
