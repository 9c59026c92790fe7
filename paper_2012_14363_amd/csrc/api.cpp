// C ABI entry points (see include/tp_pack.h for the contract of each).
#include "tp_pack.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "canon.hpp"
#include "kernels.hpp"
#include "plan.hpp"
#include "status.hpp"
#include "type_tree.hpp"

namespace {

using namespace tp;

std::atomic<int> g_max_word_log2{4};
std::atomic<int> g_nt{-1};
std::atomic<bool> g_check_buffers{true};
std::atomic<int64_t> g_max_rows_per_launch{int64_t{1} << 30};
std::atomic<int64_t> g_max_words_per_run{int64_t{1} << 30};

thread_local std::string t_last_plan;
thread_local std::string t_last_hip_error;

int register_type(int status, TypePtr node, tp_type* newtype) {
    if (status != kSuccess) return status;
    const int32_t h = HandleTable::instance().insert(std::move(node));
    if (h < 0) return kErrRange;
    *newtype = h;
    return kSuccess;
}

// Commit = Sec. 3's three phases, run once per node and cached in it.
int commit_node(const TypeNode& node) {
    std::call_once(node.commit_once, [&node] {
        StridedBlock sb;
        const int rc = canonicalize(node, &sb);
        node.commit_status = rc;
        if (rc != kSuccess) return;
        node.block = sb;
        uint64_t bits = static_cast<uint64_t>(sb.counts[0]) | static_cast<uint64_t>(sb.start < 0 ? -sb.start : sb.start);
        for (int d = 1; d < sb.ndims; ++d)
            bits |= static_cast<uint64_t>(sb.strides[d] < 0 ? -sb.strides[d] : sb.strides[d]);
        bits |= static_cast<uint64_t>(node.extent());
        node.type_align_log2 = bits ? std::min(4, __builtin_ctzll(bits)) : 4;
        node.committed = true;
    });
    return node.commit_status;
}

// A handle's node if it may be used for data movement: committed, or predefined
// (predefined types count as committed from the start and are committed on first use).
TypePtr committed_node(tp_type t) {
    TypePtr node = HandleTable::instance().lookup(t);
    if (!node) return nullptr;
    if (node->kind == Kind::Named && commit_node(*node) != kSuccess) return nullptr;
    return node->committed ? node : nullptr;
}

// Resolves a data pointer to an address the GPU can use.  `allow_host`: pinned,
// GPU-mapped host memory is acceptable (the contiguous side only).
int resolve_pointer(const void* ptr, bool allow_host, const char** device_view) {
    if (!g_check_buffers.load(std::memory_order_relaxed)) {
        *device_view = static_cast<const char*>(ptr);
        return kSuccess;
    }
    hipPointerAttribute_t attr;
    std::memset(&attr, 0, sizeof attr);
    const hipError_t e = hipPointerGetAttributes(&attr, ptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();  // an unknown pointer is reported as an error by some runtimes: clear it
        if (e == hipErrorInvalidValue) return kErrBuffer;
        t_last_hip_error = hipGetErrorString(e);
        return kErrOther;
    }
    switch (attr.type) {
    case hipMemoryTypeDevice:
    case hipMemoryTypeManaged:
        *device_view = static_cast<const char*>(ptr);
        return kSuccess;
    case hipMemoryTypeHost:
        if (!allow_host || !attr.devicePointer) return kErrBuffer;
        *device_view = static_cast<const char*>(attr.devicePointer);
        return kSuccess;
    default:
        return kErrBuffer;  // pageable host memory
    }
}

int transfer(bool unpack, const void* typed_buf, int64_t count, tp_type t, const void* packed_buf,
             int64_t packed_size, int64_t* position, void* hip_stream, bool synchronize) {
    if (!position) return kErrArg;
    const TypePtr node = committed_node(t);
    if (!node) return kErrType;
    if (count < 0) return kErrCount;
    if (*position < 0 || packed_size < 0) return kErrArg;
    int64_t bytes;
    if (__builtin_mul_overflow(count, node->size, &bytes)) return kErrRange;
    if (bytes > packed_size - *position) return kErrTruncate;
    t_last_plan.clear();
    if (bytes == 0) return kSuccess;
    if (!typed_buf || !packed_buf) return kErrBuffer;

    const char* typed_view = nullptr;
    const char* packed_view = nullptr;
    int rc = resolve_pointer(typed_buf, false, &typed_view);
    if (rc != kSuccess) return rc;
    rc = resolve_pointer(packed_buf, true, &packed_view);
    if (rc != kSuccess) return rc;

    PlanInput in;
    in.block = node->block;
    in.extent = node->extent();
    in.count = count;
    in.typed = typed_view;
    in.packed = const_cast<char*>(packed_view) + *position;
    in.max_word_log2 = g_max_word_log2.load(std::memory_order_relaxed);
    in.nt = g_nt.load(std::memory_order_relaxed);
    in.unpack = unpack;
    in.max_rows_per_launch = g_max_rows_per_launch.load(std::memory_order_relaxed);
    in.max_words_per_run = g_max_words_per_run.load(std::memory_order_relaxed);
    std::vector<Launch> launches;
    rc = plan_launches(in, &launches);
    if (rc != kSuccess) return rc;
    t_last_plan = describe(launches);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (const Launch& l : launches) {
        const hipError_t e = enqueue(l, unpack, stream);
        if (e != hipSuccess) {
            t_last_hip_error = hipGetErrorString(e);
            return kErrOther;
        }
    }
    if (synchronize) {
        const hipError_t e = hipStreamSynchronize(stream);
        if (e != hipSuccess) {
            t_last_hip_error = hipGetErrorString(e);
            return kErrOther;
        }
    }
    *position += bytes;
    return kSuccess;
}

}  // namespace

extern "C" {

int tp_type_contiguous(int count, tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    return register_type(make_contiguous(count, o, &n), n, newtype);
}

int tp_type_vector(int count, int blocklength, int stride, tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    return register_type(make_vector(count, blocklength, stride, false, o, &n), n, newtype);
}

int tp_type_create_hvector(int count, int blocklength, int64_t stride_bytes, tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    return register_type(make_vector(count, blocklength, stride_bytes, true, o, &n), n, newtype);
}

int tp_type_create_subarray(int ndims, const int sizes[], const int subsizes[], const int starts[], int order,
                            tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    return register_type(make_subarray(ndims, sizes, subsizes, starts, order, o, &n), n, newtype);
}

int tp_type_commit(tp_type* t) {
    if (!t) return kErrArg;
    const TypePtr node = HandleTable::instance().lookup(*t);
    if (!node) return kErrType;
    return commit_node(*node);
}

int tp_type_free(tp_type* t) {
    if (!t) return kErrArg;
    if (!HandleTable::instance().erase(*t)) return kErrType;
    *t = TP_TYPE_NULL;
    return kSuccess;
}

int tp_type_size(tp_type t, int64_t* size) {
    if (!size) return kErrArg;
    const TypePtr node = HandleTable::instance().lookup(t);
    if (!node) return kErrType;
    *size = node->size;
    return kSuccess;
}

int tp_type_get_extent(tp_type t, int64_t* lb, int64_t* extent) {
    if (!lb || !extent) return kErrArg;
    const TypePtr node = HandleTable::instance().lookup(t);
    if (!node) return kErrType;
    *lb = node->lb;
    *extent = node->extent();
    return kSuccess;
}

int tp_pack_size(int incount, tp_type t, int64_t* size) {
    if (!size) return kErrArg;
    const TypePtr node = HandleTable::instance().lookup(t);
    if (!node) return kErrType;
    if (incount < 0) return kErrCount;
    int64_t bytes;
    if (__builtin_mul_overflow(static_cast<int64_t>(incount), node->size, &bytes)) return kErrRange;
    *size = bytes;
    return kSuccess;
}

int tp_pack(const void* inbuf, int incount, tp_type t, void* outbuf, int64_t outsize, int64_t* position,
            void* hip_stream) {
    return transfer(false, inbuf, incount, t, outbuf, outsize, position, hip_stream, true);
}

int tp_unpack(const void* inbuf, int64_t insize, int64_t* position, void* outbuf, int outcount, tp_type t,
              void* hip_stream) {
    return transfer(true, outbuf, outcount, t, inbuf, insize, position, hip_stream, true);
}

int tp_pack_async(const void* inbuf, int incount, tp_type t, void* outbuf, int64_t outsize, int64_t* position,
                  void* hip_stream) {
    return transfer(false, inbuf, incount, t, outbuf, outsize, position, hip_stream, false);
}

int tp_unpack_async(const void* inbuf, int64_t insize, int64_t* position, void* outbuf, int outcount, tp_type t,
                    void* hip_stream) {
    return transfer(true, outbuf, outcount, t, inbuf, insize, position, hip_stream, false);
}

int tp_type_get_strided_block(tp_type t, int* ndims, int64_t* start, int64_t counts[], int64_t strides[]) {
    if (!ndims || !start || !counts || !strides) return kErrArg;
    const TypePtr node = committed_node(t);
    if (!node) return kErrType;
    const StridedBlock& sb = node->block;
    *ndims = sb.ndims;
    *start = sb.start;
    for (int d = 0; d < sb.ndims; ++d) {
        counts[d] = sb.counts[d];
        strides[d] = sb.strides[d];
    }
    return kSuccess;
}

int tp_set_override(const char* key, const char* value) {
    if (!key || !value) return kErrArg;
    char* end = nullptr;
    const long long v = std::strtoll(value, &end, 10);
    if (end == value || *end != '\0') return kErrArg;
    if (!std::strcmp(key, "word")) {
        int log2 = 4;
        switch (v) {
        case 0: log2 = 4; break;
        case 1: log2 = 0; break;
        case 2: log2 = 1; break;
        case 4: log2 = 2; break;
        case 8: log2 = 3; break;
        case 16: log2 = 4; break;
        default: return kErrArg;
        }
        g_max_word_log2.store(log2);
        return kSuccess;
    }
    if (!std::strcmp(key, "nt")) {
        if (v < -1 || v > 3) return kErrArg;
        g_nt.store(static_cast<int>(v));
        return kSuccess;
    }
    if (!std::strcmp(key, "check_buffers")) {
        if (v != 0 && v != 1) return kErrArg;
        g_check_buffers.store(v == 1);
        return kSuccess;
    }
    if (!std::strcmp(key, "max_rows_per_launch")) {
        if (v < 1 || v > (1ll << 30)) return kErrArg;
        g_max_rows_per_launch.store(v);
        return kSuccess;
    }
    if (!std::strcmp(key, "max_words_per_run")) {
        if (v < 1 || v > (1ll << 30)) return kErrArg;
        g_max_words_per_run.store(v);
        return kSuccess;
    }
    return kErrArg;
}

const char* tp_last_plan(void) { return t_last_plan.c_str(); }

const char* tp_error_string(int code) {
    switch (code) {
    case kSuccess: return "success";
    case kErrType: return "invalid datatype handle, or datatype not committed";
    case kErrCount: return "negative count";
    case kErrArg: return "invalid argument";
    case kErrTruncate: return "packed data does not fit the contiguous buffer";
    case kErrBuffer: return "null buffer, or memory the GPU cannot address";
    case kErrOther: return t_last_hip_error.empty() ? "HIP runtime failure" : t_last_hip_error.c_str();
    case kErrRange: return "size or dimension count out of range";
    default: return "unknown error code";
    }
}

}  // extern "C"
