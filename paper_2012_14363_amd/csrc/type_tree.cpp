#include "type_tree.hpp"

#include <algorithm>

#include "status.hpp"

namespace tp {

namespace {

bool mul_ok(int64_t a, int64_t b, int64_t* r) { return !__builtin_mul_overflow(a, b, r); }
bool add_ok(int64_t a, int64_t b, int64_t* r) { return !__builtin_add_overflow(a, b, r); }

// Bounds of `count` copies of a span [lb, ub) placed `stride` bytes apart (count >= 1).
bool replicate_span(int64_t count, int64_t stride, int64_t* lb, int64_t* ub) {
    int64_t last;
    if (!mul_ok(count - 1, stride, &last)) return false;
    const int64_t lo = std::min<int64_t>(0, last), hi = std::max<int64_t>(0, last);
    return add_ok(*lb, lo, lb) && add_ok(*ub, hi, ub);
}

}  // namespace

int make_named(int64_t size_bytes, TypePtr* out) {
    auto n = std::make_shared<TypeNode>();
    n->kind = Kind::Named;
    n->size = size_bytes;
    n->lb = 0;
    n->ub = size_bytes;
    *out = std::move(n);
    return kSuccess;
}

int make_contiguous(int64_t count, const TypePtr& old, TypePtr* out) {
    if (count < 0) return kErrCount;
    auto n = std::make_shared<TypeNode>();
    n->kind = Kind::Contiguous;
    n->count = count;
    n->old = old;
    if (!mul_ok(count, old->size, &n->size)) return kErrRange;
    if (count > 0) {
        n->lb = old->lb;
        n->ub = old->ub;
        if (!replicate_span(count, old->extent(), &n->lb, &n->ub)) return kErrRange;
    }
    *out = std::move(n);
    return kSuccess;
}

int make_vector(int64_t count, int64_t blocklength, int64_t stride, bool stride_in_bytes, const TypePtr& old,
                TypePtr* out) {
    if (count < 0 || blocklength < 0) return kErrCount;
    auto n = std::make_shared<TypeNode>();
    n->kind = stride_in_bytes ? Kind::Hvector : Kind::Vector;
    n->count = count;
    n->blocklength = blocklength;
    n->stride = stride;
    n->old = old;
    int64_t per_block;
    if (!mul_ok(blocklength, old->size, &per_block) || !mul_ok(count, per_block, &n->size)) return kErrRange;
    if (count > 0 && blocklength > 0) {
        int64_t stride_bytes = stride;
        if (!stride_in_bytes && !mul_ok(stride, old->extent(), &stride_bytes)) return kErrRange;
        n->lb = old->lb;
        n->ub = old->ub;
        if (!replicate_span(blocklength, old->extent(), &n->lb, &n->ub)) return kErrRange;
        if (!replicate_span(count, stride_bytes, &n->lb, &n->ub)) return kErrRange;
    }
    *out = std::move(n);
    return kSuccess;
}

int make_subarray(int ndims, const int* sizes, const int* subsizes, const int* starts, int order, const TypePtr& old,
                  TypePtr* out) {
    if (ndims < 1 || ndims > kMaxDims || !sizes || !subsizes || !starts) return kErrArg;
    if (order != 0 && order != 1) return kErrArg;
    auto n = std::make_shared<TypeNode>();
    n->kind = Kind::Subarray;
    n->order = order;
    n->old = old;
    int64_t total = 1, picked = 1;
    for (int d = 0; d < ndims; ++d) {
        const int64_t sz = sizes[d], sub = subsizes[d], st = starts[d];
        if (sz < 1 || sub < 0 || sub > sz || st < 0 || st > sz - sub) return kErrArg;
        n->sizes.push_back(sz);
        n->subsizes.push_back(sub);
        n->starts.push_back(st);
        if (!mul_ok(total, sz, &total) || !mul_ok(picked, sub, &picked)) return kErrRange;
    }
    if (!mul_ok(picked, old->size, &n->size)) return kErrRange;
    n->lb = 0;
    if (!mul_ok(total, old->extent(), &n->ub)) return kErrRange;
    *out = std::move(n);
    return kSuccess;
}

// ------------------------------------------------------------------ handle table
HandleTable::HandleTable() {
    static const int64_t kNamedSizes[] = {1, 1, 1, 1, 2, 2, 4, 4, 8, 8, 4, 8};
    for (int64_t s : kNamedSizes) {
        TypePtr t;
        make_named(s, &t);
        Slot slot;
        slot.node = std::move(t);
        slots_.push_back(std::move(slot));
    }
}

HandleTable& HandleTable::instance() {
    static HandleTable table;
    return table;
}

int32_t HandleTable::insert(TypePtr node) {
    std::lock_guard<std::mutex> lock(mu_);
    uint32_t idx;
    if (!free_.empty()) {
        idx = free_.back();
        free_.pop_back();
    } else {
        if (slots_.size() >= (1u << kIndexBits)) return -1;
        idx = static_cast<uint32_t>(slots_.size());
        slots_.emplace_back();
    }
    slots_[idx].node = std::move(node);
    return static_cast<int32_t>((slots_[idx].generation << kIndexBits) | idx);
}

TypePtr HandleTable::lookup(int32_t handle) const {
    if (handle < 0) return nullptr;
    const uint32_t idx = static_cast<uint32_t>(handle) & ((1u << kIndexBits) - 1);
    const uint32_t gen = static_cast<uint32_t>(handle) >> kIndexBits;
    std::lock_guard<std::mutex> lock(mu_);
    if (idx >= slots_.size() || slots_[idx].generation != gen) return nullptr;
    return slots_[idx].node;
}

bool HandleTable::erase(int32_t handle) {
    if (handle < 12) return false;  // negative, or one of the predefined types
    const uint32_t idx = static_cast<uint32_t>(handle) & ((1u << kIndexBits) - 1);
    const uint32_t gen = static_cast<uint32_t>(handle) >> kIndexBits;
    std::lock_guard<std::mutex> lock(mu_);
    if (idx >= slots_.size() || slots_[idx].generation != gen || !slots_[idx].node) return false;
    slots_[idx].node.reset();
    slots_[idx].generation = (slots_[idx].generation + 1) & ((1u << (31 - kIndexBits)) - 1);
    free_.push_back(idx);
    return true;
}

}  // namespace tp
