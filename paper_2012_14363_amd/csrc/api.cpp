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

#include "buffer_map.hpp"
#include "canon.hpp"
#include "kernels.hpp"
#include "plan.hpp"
#include "resource_cache.hpp"
#include "status.hpp"
#include "transfer.hpp"
#include "type_tree.hpp"

namespace {

using namespace tp;

std::atomic<int> g_max_word_log2{4};
std::atomic<int> g_nt{-1};
std::atomic<bool> g_check_buffers{true};
std::atomic<bool> g_narrow_partial_rows{true};
std::atomic<int> g_max_ur{-1};
std::atomic<int> g_unpack_rule{1};
std::atomic<int> g_stage{-1};
std::atomic<int64_t> g_stage_bytes{int64_t{16} << 20};
std::atomic<int> g_stage_grid{0};
std::atomic<int> g_grid{0};
std::atomic<bool> g_allow_xpose{true};
std::atomic<int64_t> g_max_rows_per_launch{int64_t{1} << 30};
std::atomic<int64_t> g_max_words_per_run{int64_t{1} << 30};

// What the calling thread's last pack/unpack enqueued; formatted only when tp_last_plan() asks.
struct LastPlan {
    std::vector<BatchParams> batches;
    std::vector<Launch> launches;
    std::string text;
    void clear() {
        batches.clear();
        launches.clear();
    }
};
thread_local LastPlan t_last_plan;
thread_local std::string t_last_hip_error;

int register_type(TypePtr node, tp_type* newtype) {
    const int32_t h = HandleTable::instance().insert(std::move(node));
    if (h < 0) return kErrRange;
    *newtype = h;
    return kSuccess;
}

// A handle's node if it may be used for data movement: committed, or predefined
// (predefined types count as committed from the start and are committed on first use).
TypePtr committed_node(tp_type t) {
    TypePtr node = HandleTable::instance().lookup(t);
    if (!node) return nullptr;
    if (node->kind == Kind::Named && commit(*node) != kSuccess) return nullptr;
    return node->committed.load(std::memory_order_acquire) ? node : nullptr;
}

// BufferMap's query: the allocation that holds `ptr`, from the library's own leases or else from
// the runtime.
int query_memory(const void* ptr, MemRange* range) {
    const uintptr_t a = reinterpret_cast<uintptr_t>(ptr);
    // buffers leased from the library's own cache are known without asking the runtime
    int kind = 0;
    int64_t room = 0;
    const char* view = nullptr;
    if (library_resources().find_leased(ptr, &kind, &view, &room)) {
        range->lo = a;
        range->hi = a + static_cast<uintptr_t>(room);
        range->host = kind != kResDevice;
        range->view_delta = view - static_cast<const char*>(ptr);
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
        range->host = false;
        range->view_delta = 0;
        break;
    case hipMemoryTypeHost:
        if (!attr.devicePointer) return kErrBuffer;
        range->host = true;
        range->view_delta = static_cast<const char*>(attr.devicePointer) - static_cast<const char*>(ptr);
        break;
    default:
        return kErrBuffer;  // pageable host memory
    }
    // the allocation's bounds; where the runtime does not tell, only `ptr` itself is known
    void* base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void*>(ptr)) == hipSuccess && size > 0) {
        range->lo = reinterpret_cast<uintptr_t>(base);
        range->hi = range->lo + size;
    } else {
        (void)hipGetLastError();
        range->lo = a;
        range->hi = a + 1;
    }
    return kSuccess;
}

BufferMap::Query buffer_query() { return g_check_buffers.load(std::memory_order_relaxed) ? query_memory : nullptr; }

// Checks of one pack/unpack request that need no device: handle, count, fit, null buffers.
// On success *bytes is what the request moves and *node its datatype.
int check_request(const void* typed_buf, int64_t count, tp_type t, const void* packed_buf, int64_t packed_size,
                  int64_t position, TypePtr* node, int64_t* bytes) {
    *node = committed_node(t);
    if (!*node) return kErrType;
    if (count < 0) return kErrCount;
    if (__builtin_mul_overflow(count, (*node)->size, bytes)) return kErrRange;
    if (*bytes > packed_size - position) return kErrTruncate;
    if (*bytes > 0 && (!typed_buf || !packed_buf)) return kErrBuffer;
    return kSuccess;
}

// Displacements, from the origin, of the lowest and the highest byte that `count` objects of a
// committed non-empty type select.
int data_span(const TypeNode& node, int64_t count, int64_t* lo, int64_t* hi) {
    const StridedBlock& sb = node.block;
    *lo = *hi = sb.start;
    auto widen = [&](int64_t steps, int64_t stride) {
        int64_t reach;
        if (__builtin_mul_overflow(steps, stride, &reach)) return false;
        return !__builtin_add_overflow(reach < 0 ? *lo : *hi, reach, reach < 0 ? lo : hi);
    };
    for (int d = 1; d < sb.ndims; ++d)
        if (!widen(sb.counts[d] - 1, sb.strides[d])) return kErrRange;
    if (!widen(count - 1, node.extent())) return kErrRange;
    if (__builtin_add_overflow(*hi, sb.counts[0] - 1, hi)) return kErrRange;
    return kSuccess;
}

// Checks the buffers of a request that has passed check_request and appends its planned launches
// to `launches`.  `packed` is the contiguous buffer as the caller passed it.
int plan_request(bool unpack, const TypeNode& node, const void* typed_buf, int64_t count, const void* packed,
                 int64_t position, BufferMap* memory, std::vector<Launch>* launches, bool batched = false) {
    // Query the first selected byte, not the origin: MPI lets the origin lie outside the
    // allocation (negative strides, lower bounds above zero); the data never does.
    const char* typed = static_cast<const char*>(typed_buf);
    const char* first_byte = nullptr;
    int rc = memory->locate(typed + node.block.start, false, &first_byte);
    if (rc != kSuccess) return rc;
    const char* typed_view = first_byte - node.block.start;
    // So are the lowest and the highest byte the request touches, on both sides: a datatype that
    // runs past its buffer is reported here instead of as a GPU memory fault.  (Bytes in between
    // are not queried; an allocation boundary crossed on the way to valid memory goes unnoticed.)
    int64_t lo = 0, hi = 0;
    rc = data_span(node, count, &lo, &hi);
    if (rc != kSuccess) return rc;
    if ((rc = memory->check(typed + lo, false)) != kSuccess) return rc;
    if ((rc = memory->check(typed + hi, false)) != kSuccess) return rc;
    const char* packed_first = static_cast<const char*>(packed) + position;
    const char* packed_view = nullptr;
    bool packed_on_host = false;
    if ((rc = memory->locate(packed_first, true, &packed_view, &packed_on_host)) != kSuccess) return rc;
    if ((rc = memory->check(packed_first + count * node.size - 1, true)) != kSuccess) return rc;
    PlanInput in;
    in.block = node.block;
    in.extent = node.extent();
    in.count = count;
    in.typed = typed_view;
    in.packed = const_cast<char*>(packed_view);
    in.unpack = unpack;
    in.packed_on_host = packed_on_host;
    in.batched = batched;
    in.narrow_partial_rows = g_narrow_partial_rows.load(std::memory_order_relaxed);
    in.max_ur = g_max_ur.load(std::memory_order_relaxed);
    in.unpack_rule = g_unpack_rule.load(std::memory_order_relaxed);
    in.stage = g_stage.load(std::memory_order_relaxed);
    in.stage_bytes = g_stage_bytes.load(std::memory_order_relaxed);
    in.stage_grid = g_stage_grid.load(std::memory_order_relaxed);
    in.grid = g_grid.load(std::memory_order_relaxed);
    in.allow_xpose = g_allow_xpose.load(std::memory_order_relaxed);
    in.max_word_log2 = g_max_word_log2.load(std::memory_order_relaxed);
    in.nt = g_nt.load(std::memory_order_relaxed);
    in.max_rows_per_launch = g_max_rows_per_launch.load(std::memory_order_relaxed);
    in.max_words_per_run = g_max_words_per_run.load(std::memory_order_relaxed);
    std::vector<Launch> mine;
    rc = plan_launches(in, &mine);
    if (rc != kSuccess) return rc;
    launches->insert(launches->end(), mine.begin(), mine.end());
    return kSuccess;
}

int finish(hipStream_t stream, bool synchronize) {
    if (!synchronize) return kSuccess;
    const hipError_t e = hipStreamSynchronize(stream);
    if (e != hipSuccess) {
        t_last_hip_error = hipGetErrorString(e);
        return kErrOther;
    }
    return kSuccess;
}

int transfer(bool unpack, const void* typed_buf, int64_t count, tp_type t, const void* packed_buf,
             int64_t packed_size, int64_t* position, void* hip_stream, bool synchronize,
             const MemRange* vouched = nullptr) {
    if (!position) return kErrArg;
    if (*position < 0 || packed_size < 0) return kErrArg;
    t_last_plan.clear();
    BufferMap memory(buffer_query());
    if (vouched) memory.add_known(*vouched);
    TypePtr node;
    int64_t bytes = 0;
    int rc = check_request(typed_buf, count, t, packed_buf, packed_size, *position, &node, &bytes);
    if (rc != kSuccess) return rc;
    std::vector<Launch> launches;
    if (bytes > 0) {
        rc = plan_request(unpack, *node, typed_buf, count, packed_buf, *position, &memory, &launches);
        if (rc != kSuccess) return rc;
    }
    const int64_t pos = *position + bytes;
    t_last_plan.launches = launches;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (const Launch& l : launches) {
        const hipError_t e = enqueue(l, unpack, stream);
        if (e != hipSuccess) {
            t_last_hip_error = hipGetErrorString(e);
            return kErrOther;
        }
    }
    if (!launches.empty()) {
        rc = finish(stream, synchronize);
        if (rc != kSuccess) return rc;
    }
    *position = pos;
    return kSuccess;
}

// n pack (or unpack) requests sharing one contiguous buffer and one running position, enqueued
// as few launches as possible.  All requests are validated and planned before anything is enqueued.
int transfer_batch(bool unpack, int n, const void* const* typed_bufs, const int* counts, const tp_type* types,
                   const void* packed_buf, int64_t packed_size, int64_t* position, void* hip_stream,
                   bool synchronize) {
    if (!position || n < 0) return kErrArg;
    if (n > 0 && (!typed_bufs || !counts || !types)) return kErrArg;
    if (*position < 0 || packed_size < 0) return kErrArg;
    t_last_plan.clear();
    BufferMap memory(buffer_query());
    int64_t pos = *position;
    std::vector<TypePtr> nodes(static_cast<size_t>(n));
    std::vector<int64_t> offsets(static_cast<size_t>(n)), sizes(static_cast<size_t>(n));
    for (int i = 0; i < n; ++i) {  // every check that needs no device, for all requests, first
        const int rc = check_request(typed_bufs[i], counts[i], types[i], packed_buf, packed_size, pos, &nodes[i],
                                     &sizes[i]);
        if (rc != kSuccess) return rc;
        offsets[i] = pos;
        pos += sizes[i];
    }
    std::vector<Launch> launches;
    for (int i = 0; i < n; ++i) {
        if (sizes[i] == 0) continue;
        const int rc =
            plan_request(unpack, *nodes[i], typed_bufs[i], counts[i], packed_buf, offsets[i], &memory, &launches, true);
        if (rc != kSuccess) return rc;
    }
    std::vector<BatchParams> batches;
    std::vector<Launch> singles;
    make_batches(launches, &batches, &singles);
    t_last_plan.batches = batches;
    t_last_plan.launches = singles;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    for (const BatchParams& b : batches) {
        const hipError_t e = enqueue_batch(b, unpack, stream);
        if (e != hipSuccess) {
            t_last_hip_error = hipGetErrorString(e);
            return kErrOther;
        }
    }
    for (const Launch& l : singles) {
        const hipError_t e = enqueue(l, unpack, stream);
        if (e != hipSuccess) {
            t_last_hip_error = hipGetErrorString(e);
            return kErrOther;
        }
    }
    if (!launches.empty()) {
        const int rc = finish(stream, synchronize);
        if (rc != kSuccess) return rc;
    }
    *position = pos;
    return kSuccess;
}

}  // namespace

namespace tp {

int transfer_with_device_buffer(bool unpack, const void* typed_buf, int64_t count, tp_type t, void* device_buf,
                                int64_t size, int64_t* position, hipStream_t stream) {
    if (!device_buf || size < 0) return kErrArg;
    MemRange mine;
    mine.lo = reinterpret_cast<uintptr_t>(device_buf);
    mine.hi = mine.lo + static_cast<uintptr_t>(size);
    return transfer(unpack, typed_buf, count, t, device_buf, size, position, stream, false, &mine);
}

int copy_device_buffer_to_packed(const void* device_src, int64_t bytes, void* packed_buf, int64_t packed_size,
                                 int64_t position, hipStream_t stream) {
    if (bytes < 0 || position < 0 || packed_size < 0) return kErrArg;
    if (bytes > packed_size - position) return kErrTruncate;
    if (bytes == 0) return kSuccess;
    if (!device_src || !packed_buf) return kErrBuffer;
    BufferMap memory(buffer_query());
    const char* first = static_cast<const char*>(packed_buf) + position;
    const char* view = nullptr;
    bool on_host = false;
    int rc = memory.locate(first, true, &view, &on_host);
    if (rc != kSuccess) return rc;
    if ((rc = memory.check(first + bytes - 1, true)) != kSuccess) return rc;
    PlanInput in;   // one run of `bytes`: the fully dense datatype
    in.block.ndims = 1;
    in.block.start = 0;
    in.block.counts[0] = bytes;
    in.block.strides[0] = 1;
    in.extent = bytes;
    in.count = 1;
    in.typed = static_cast<const char*>(device_src);
    in.packed = const_cast<char*>(view);
    in.packed_on_host = on_host;
    std::vector<Launch> launches;
    rc = plan_launches(in, &launches);
    if (rc != kSuccess) return rc;
    for (const Launch& l : launches) {
        const hipError_t e = enqueue(l, false, stream);
        if (e != hipSuccess) {
            t_last_hip_error = hipGetErrorString(e);
            return kErrOther;
        }
    }
    return kSuccess;
}

}  // namespace tp

extern "C" {

int tp_type_contiguous(int count, tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    const int rc = make_contiguous(count, o, &n);
    if (rc != kSuccess) return rc;
    return register_type(std::move(n), newtype);
}

int tp_type_vector(int count, int blocklength, int stride, tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    const int rc = make_vector(count, blocklength, stride, false, o, &n);
    if (rc != kSuccess) return rc;
    return register_type(std::move(n), newtype);
}

int tp_type_create_hvector(int count, int blocklength, int64_t stride_bytes, tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    const int rc = make_vector(count, blocklength, stride_bytes, true, o, &n);
    if (rc != kSuccess) return rc;
    return register_type(std::move(n), newtype);
}

int tp_type_create_subarray(int ndims, const int sizes[], const int subsizes[], const int starts[], int order,
                            tp_type old, tp_type* newtype) {
    if (!newtype) return kErrArg;
    const TypePtr o = HandleTable::instance().lookup(old);
    if (!o) return kErrType;
    TypePtr n;
    const int rc = make_subarray(ndims, sizes, subsizes, starts, order, o, &n);
    if (rc != kSuccess) return rc;
    return register_type(std::move(n), newtype);
}

int tp_type_commit(tp_type* t) {
    if (!t) return kErrArg;
    const TypePtr node = HandleTable::instance().lookup(*t);
    if (!node) return kErrType;
    return commit(*node);
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

int tp_pack_batch(int n, const void* const inbufs[], const int incounts[], const tp_type types[], void* outbuf,
                  int64_t outsize, int64_t* position, void* hip_stream) {
    return transfer_batch(false, n, inbufs, incounts, types, outbuf, outsize, position, hip_stream, true);
}

int tp_unpack_batch(int n, const void* inbuf, int64_t insize, int64_t* position, void* const outbufs[],
                    const int outcounts[], const tp_type types[], void* hip_stream) {
    return transfer_batch(true, n, outbufs, outcounts, types, inbuf, insize, position, hip_stream, true);
}

int tp_pack_batch_async(int n, const void* const inbufs[], const int incounts[], const tp_type types[], void* outbuf,
                        int64_t outsize, int64_t* position, void* hip_stream) {
    return transfer_batch(false, n, inbufs, incounts, types, outbuf, outsize, position, hip_stream, false);
}

int tp_unpack_batch_async(int n, const void* inbuf, int64_t insize, int64_t* position, void* const outbufs[],
                          const int outcounts[], const tp_type types[], void* hip_stream) {
    return transfer_batch(true, n, outbufs, outcounts, types, inbuf, insize, position, hip_stream, false);
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
        if ((v < -1 || v > 3) && v != 6 && v != 7) return kErrArg;
        g_nt.store(static_cast<int>(v));
        return kSuccess;
    }
    if (!std::strcmp(key, "ur")) {
        if (v != -1 && v != 1 && v != 4) return kErrArg;
        g_max_ur.store(static_cast<int>(v));
        return kSuccess;
    }
    if (!std::strcmp(key, "stage")) {
        if (v < -1 || v > 1) return kErrArg;
        g_stage.store(static_cast<int>(v));
        return kSuccess;
    }
    if (!std::strcmp(key, "stage_bytes")) {
        if (v < 4096 || v > (1ll << 30)) return kErrArg;
        g_stage_bytes.store(v);
        return kSuccess;
    }
    if (!std::strcmp(key, "stage_grid")) {
        if (v < 0 || v > (1ll << 20)) return kErrArg;
        g_stage_grid.store(static_cast<int>(v));
        return kSuccess;
    }
    if (!std::strcmp(key, "grid")) {
        if (v < 0 || v > (1ll << 20)) return kErrArg;
        g_grid.store(static_cast<int>(v));
        return kSuccess;
    }
    if (!std::strcmp(key, "unpack_rule")) {
        if (v != 0 && v != 1) return kErrArg;
        g_unpack_rule.store(static_cast<int>(v));
        return kSuccess;
    }
    if (!std::strcmp(key, "xpose")) {
        if (v != 0 && v != 1) return kErrArg;
        g_allow_xpose.store(v == 1);
        return kSuccess;
    }
    if (!std::strcmp(key, "narrow_partial_rows")) {
        if (v != 0 && v != 1) return kErrArg;
        g_narrow_partial_rows.store(v == 1);
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

const char* tp_last_plan(void) {
    t_last_plan.text = describe(t_last_plan.batches) + describe(t_last_plan.launches);
    return t_last_plan.text.c_str();
}

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
