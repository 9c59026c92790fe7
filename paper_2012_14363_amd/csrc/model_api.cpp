// C ABI of the measured performance model and of the host-delivery calls that use it
// (see include/tp_pack.h).  Paper Sec. 4 (Eq. 1-3) and Sec. 6.3.
#include "tp_pack.h"

#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstring>
#include <fstream>
#include <sstream>
#include <vector>

#include "model.hpp"
#include "resource_cache.hpp"
#include "status.hpp"

namespace {

using namespace tp;
using Clock = std::chrono::steady_clock;

double seconds_since(Clock::time_point t0) { return std::chrono::duration<double>(Clock::now() - t0).count(); }

// Median wall time of `fn` (which must include its own synchronization): 2 warm-ups, then
// up to `reps` timed calls, fewer once a single call takes longer than 20 ms.
template <class F>
double median_time(F&& fn, int reps, int* status) {
    for (int i = 0; i < 2; ++i) {
        *status = fn();
        if (*status != kSuccess) return 0.0;
    }
    std::vector<double> t;
    for (int i = 0; i < reps; ++i) {
        const auto t0 = Clock::now();
        *status = fn();
        if (*status != kSuccess) return 0.0;
        t.push_back(seconds_since(t0));
        if (t.back() > 0.02 && t.size() >= 3) break;
    }
    std::sort(t.begin(), t.end());
    return t[t.size() / 2];
}

struct Buffers {
    char* typed = nullptr;
    char* packed = nullptr;
    char* pinned = nullptr;
    ~Buffers() {
        if (typed) (void)hipFree(typed);
        if (packed) (void)hipFree(packed);
        if (pinned) (void)hipHostFree(pinned);
    }
};

// Contiguous block length the model is indexed by: the canonical run length, or the whole
// message when the type is dense.
int model_key(tp_type t, int count, int64_t* bytes, int64_t* block) {
    int64_t size;
    int rc = tp_pack_size(count, t, &size);
    if (rc != kSuccess) return rc;
    int nd;
    int64_t start, counts[TP_MAX_DIMS], strides[TP_MAX_DIMS];
    rc = tp_type_get_strided_block(t, &nd, &start, counts, strides);
    if (rc != kSuccess) return rc;
    *bytes = size;
    *block = nd > 1 ? counts[0] : std::max<int64_t>(size, 1);
    return kSuccess;
}

// The device buffer of a staged transfer: the caller's, or with none given a lease from the
// library's resource cache that ends with the call (which has synchronized by then).
struct Staging {
    void* ptr = nullptr;
    int64_t size = 0;
    bool leased = false;
    hipStream_t stream = nullptr;
    bool drained = false;  // set once the stream has been waited for after the last use of ptr
    int take(void* callers, int64_t callers_size, int64_t bytes, hipStream_t s) {
        stream = s;
        if (callers) {
            ptr = callers;
            size = callers_size;
            return kSuccess;
        }
        const int rc = library_resources().acquire(kResDevice, bytes, &ptr);
        if (rc != kSuccess) return rc;
        size = bytes;
        leased = true;
        return kSuccess;
    }
    ~Staging() {
        if (!leased) return;
        // an error path may leave a copy or kernel in flight: the next holder must not see it
        if (!drained) (void)hipStreamSynchronize(stream);
        (void)library_resources().release(kResDevice, ptr);
    }
};

}  // namespace

extern "C" {

int tp_model_measure(void* hip_stream) {
    static const int64_t kSizes[] = {64, 1024, 16384, 262144, 4194304};
    static const int64_t kBlocks[] = {1, 4, 16, 64, 256, 1024, 4096};
    const int ns = static_cast<int>(sizeof kSizes / sizeof kSizes[0]);
    const int nb = static_cast<int>(sizeof kBlocks / sizeof kBlocks[0]);
    const int64_t max_size = kSizes[ns - 1];
    const int64_t typed_bytes = max_size * 512 + 8192;  // rows of 1 byte at 512-byte pitch
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    Buffers buf;
    if (hipMalloc(reinterpret_cast<void**>(&buf.typed), static_cast<size_t>(typed_bytes)) != hipSuccess ||
        hipMalloc(reinterpret_cast<void**>(&buf.packed), static_cast<size_t>(max_size)) != hipSuccess ||
        hipHostMalloc(reinterpret_cast<void**>(&buf.pinned), static_cast<size_t>(max_size), hipHostMallocDefault) !=
            hipSuccess) {
        (void)hipGetLastError();
        return kErrOther;
    }
    if (hipMemsetAsync(buf.typed, 0x5A, static_cast<size_t>(typed_bytes), stream) != hipSuccess ||
        hipMemsetAsync(buf.packed, 0x3C, static_cast<size_t>(max_size), stream) != hipSuccess ||
        hipStreamSynchronize(stream) != hipSuccess)
        return kErrOther;
    std::memset(buf.pinned, 0x77, static_cast<size_t>(max_size));

    ModelTable tb;
    for (int s = 0; s < ns; ++s) tb.sizes.push_back(static_cast<double>(kSizes[s]));
    for (int b = 0; b < nb; ++b) tb.blocks.push_back(static_cast<double>(kBlocks[b]));
    for (auto& g : tb.grid) g.assign(static_cast<size_t>(ns) * nb, 0.0);
    for (auto& c : tb.copy) c.assign(static_cast<size_t>(ns), 0.0);

    int status = kSuccess;
    for (int s = 0; s < ns; ++s) {
        const int64_t size = kSizes[s];
        for (int b = 0; b < nb; ++b) {
            // 2D object of `size` bytes in runs of `block` bytes; 512-byte pitch as in the paper's
            // measurements, doubled pitch once the run no longer fits it
            const int64_t block = std::min(kBlocks[b], size);
            const int64_t pitch = std::max<int64_t>(512, 2 * block);
            const int64_t rows = size / block;
            if (rows * pitch > typed_bytes) return kErrRange;
            tp_type t;
            int rc = tp_type_vector(static_cast<int>(rows), static_cast<int>(block), static_cast<int>(pitch), TP_BYTE, &t);
            if (rc != kSuccess) return rc;
            rc = tp_type_commit(&t);
            if (rc != kSuccess) {
                tp_type_free(&t);
                return rc;
            }
            const int reps = size >= (1 << 20) ? 7 : 15;
            const size_t at = static_cast<size_t>(s) * nb + b;
            auto pack_to = [&](char* out) {
                return [&, out]() { int64_t pos = 0; return tp_pack(buf.typed, 1, t, out, size, &pos, hip_stream); };
            };
            auto unpack_from = [&](char* in) {
                return [&, in]() { int64_t pos = 0; return tp_unpack(in, size, &pos, buf.typed, 1, t, hip_stream); };
            };
            tb.grid[kGpuPack][at] = median_time(pack_to(buf.packed), reps, &status);
            if (status == kSuccess) tb.grid[kGpuUnpack][at] = median_time(unpack_from(buf.packed), reps, &status);
            if (status == kSuccess) tb.grid[kHostPack][at] = median_time(pack_to(buf.pinned), reps, &status);
            if (status == kSuccess) tb.grid[kHostUnpack][at] = median_time(unpack_from(buf.pinned), reps, &status);
            tp_type_free(&t);
            if (status != kSuccess) return status;
        }
        auto copy = [&](void* dst, const void* src, hipMemcpyKind kind) {
            return [=]() {
                if (hipMemcpyAsync(dst, src, static_cast<size_t>(size), kind, stream) != hipSuccess) return int(kErrOther);
                return hipStreamSynchronize(stream) == hipSuccess ? int(kSuccess) : int(kErrOther);
            };
        };
        tb.copy[0][static_cast<size_t>(s)] = median_time(copy(buf.pinned, buf.packed, hipMemcpyDeviceToHost), 15, &status);
        if (status == kSuccess)
            tb.copy[1][static_cast<size_t>(s)] = median_time(copy(buf.packed, buf.pinned, hipMemcpyHostToDevice), 15, &status);
        if (status != kSuccess) return status;
    }
    Model::instance().set(std::move(tb));
    return kSuccess;
}

int tp_model_save(const char* path) {
    if (!path) return kErrArg;
    if (!Model::instance().loaded()) return kErrArg;
    std::ofstream f(path);
    if (!f) return kErrOther;
    f << serialize(Model::instance().table());
    return f.good() ? kSuccess : kErrOther;
}

int tp_model_load(const char* path) {
    if (!path) return kErrArg;
    std::ifstream f(path);
    if (!f) return kErrOther;
    std::stringstream ss;
    ss << f.rdbuf();
    ModelTable tb;
    if (!parse(ss.str(), &tb)) return kErrArg;
    Model::instance().set(std::move(tb));
    return kSuccess;
}

int tp_model_query(tp_type t, int count, tp_model_times* out) {
    if (!out) return kErrArg;
    int64_t bytes, block;
    const int rc = model_key(t, count, &bytes, &block);
    if (rc != kSuccess) return rc;
    ModelTimes m;
    if (!Model::instance().query(bytes, block, &m)) return kErrArg;
    out->gpu_pack = m.t[kGpuPack];
    out->gpu_unpack = m.t[kGpuUnpack];
    out->host_pack = m.t[kHostPack];
    out->host_unpack = m.t[kHostUnpack];
    out->d2h = m.t[kD2H];
    out->h2d = m.t[kH2D];
    return kSuccess;
}

int tp_model_select(tp_type t, int count, double t_cpu_cpu, double t_gpu_gpu, int* method, double times[3]) {
    if (!method) return kErrArg;
    int64_t bytes, block;
    const int rc = model_key(t, count, &bytes, &block);
    if (rc != kSuccess) return rc;
    ModelTimes m;
    if (!Model::instance().query(bytes, block, &m)) return kErrArg;
    double local[3];
    *method = select_method(m, t_cpu_cpu, t_gpu_gpu, times ? times : local);
    return kSuccess;
}

int tp_pack_host(const void* inbuf, int incount, tp_type t, void* host_outbuf, int64_t outsize, int64_t* position,
                 void* staging, int64_t staging_size, int method, void* hip_stream, int* method_used) {
    if (!position) return kErrArg;
    if (method != TP_METHOD_AUTO && method != TP_METHOD_ONESHOT && method != TP_METHOD_STAGED) return kErrArg;
    int64_t bytes;
    int rc = tp_pack_size(incount, t, &bytes);
    if (rc != kSuccess) return rc;
    const bool can_stage = staging == nullptr || staging_size >= bytes;
    if (method == TP_METHOD_STAGED && !can_stage) return kErrArg;
    if (method == TP_METHOD_AUTO) {
        method = TP_METHOD_ONESHOT;
        tp_model_times m;
        if (can_stage && tp_model_query(t, incount, &m) == kSuccess && m.gpu_pack + m.d2h < m.host_pack)
            method = TP_METHOD_STAGED;
    }
    if (method == TP_METHOD_ONESHOT) {
        rc = tp_pack(inbuf, incount, t, host_outbuf, outsize, position, hip_stream);
    } else {
        if (*position < 0 || outsize < 0) return kErrArg;
        if (bytes > outsize - *position) return kErrTruncate;
        if (bytes > 0 && !host_outbuf) return kErrBuffer;
        hipStream_t stream = static_cast<hipStream_t>(hip_stream);
        Staging stage;
        rc = stage.take(staging, staging_size, bytes, stream);
        if (rc != kSuccess) return rc;
        int64_t staged = 0;
        rc = tp_pack_async(inbuf, incount, t, stage.ptr, stage.size, &staged, hip_stream);
        if (rc != kSuccess) return rc;
        if (bytes > 0 &&
            hipMemcpyAsync(static_cast<char*>(host_outbuf) + *position, stage.ptr, static_cast<size_t>(bytes),
                           hipMemcpyDeviceToHost, stream) != hipSuccess)
            return kErrOther;
        if (hipStreamSynchronize(stream) != hipSuccess) return kErrOther;
        stage.drained = true;
        *position += bytes;
    }
    if (rc == kSuccess && method_used) *method_used = method;
    return rc;
}

int tp_unpack_host(const void* host_inbuf, int64_t insize, int64_t* position, void* outbuf, int outcount, tp_type t,
                   void* staging, int64_t staging_size, int method, void* hip_stream, int* method_used) {
    if (!position) return kErrArg;
    if (method != TP_METHOD_AUTO && method != TP_METHOD_ONESHOT && method != TP_METHOD_STAGED) return kErrArg;
    int64_t bytes;
    int rc = tp_pack_size(outcount, t, &bytes);
    if (rc != kSuccess) return rc;
    const bool can_stage = staging == nullptr || staging_size >= bytes;
    if (method == TP_METHOD_STAGED && !can_stage) return kErrArg;
    if (method == TP_METHOD_AUTO) {
        method = TP_METHOD_ONESHOT;
        tp_model_times m;
        if (can_stage && tp_model_query(t, outcount, &m) == kSuccess && m.h2d + m.gpu_unpack < m.host_unpack)
            method = TP_METHOD_STAGED;
    }
    if (method == TP_METHOD_ONESHOT) {
        rc = tp_unpack(host_inbuf, insize, position, outbuf, outcount, t, hip_stream);
    } else {
        if (*position < 0 || insize < 0) return kErrArg;
        if (bytes > insize - *position) return kErrTruncate;
        if (bytes > 0 && !host_inbuf) return kErrBuffer;
        hipStream_t stream = static_cast<hipStream_t>(hip_stream);
        Staging stage;
        rc = stage.take(staging, staging_size, bytes, stream);
        if (rc != kSuccess) return rc;
        if (bytes > 0 &&
            hipMemcpyAsync(stage.ptr, static_cast<const char*>(host_inbuf) + *position, static_cast<size_t>(bytes),
                           hipMemcpyHostToDevice, stream) != hipSuccess)
            return kErrOther;
        int64_t staged = 0;
        rc = tp_unpack(stage.ptr, bytes, &staged, outbuf, outcount, t, hip_stream);
        if (rc != kSuccess) return rc;
        stage.drained = true;  // tp_unpack has waited for the copy and its kernels (none if bytes == 0)
        *position += bytes;
    }
    if (rc == kSuccess && method_used) *method_used = method;
    return rc;
}

}  // extern "C"
