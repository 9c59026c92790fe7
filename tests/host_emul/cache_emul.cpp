// The library's resource cache (resource_cache.cpp) over the host heap, for tests only: the
// bookkeeping is the product's, the backend counts what it was asked to create and destroy and
// can be told to fail, so that reuse, size classes, trimming and the out-of-memory retry can be
// checked without a GPU.
#include <atomic>
#include <cstdint>
#include <cstdlib>
#include <thread>
#include <vector>

#include "resource_cache.hpp"

namespace {

std::atomic<int64_t> g_created[tp::kResKinds];
std::atomic<int64_t> g_destroyed[tp::kResKinds];
std::atomic<int64_t> g_live_bytes{0};
std::atomic<int> g_fail_next{0};
thread_local int t_device = 0;

bool heap_create(int kind, int /*device*/, size_t bytes, void** handle, void** gpu_view) {
    if (g_fail_next.load() > 0 && g_fail_next.fetch_sub(1) > 0) return false;
    // streams and events are opaque handles: any distinct address will do
    void* p = std::malloc(tp::is_buffer_kind(kind) ? bytes + sizeof(size_t) : 16);
    if (!p) return false;
    if (tp::is_buffer_kind(kind)) {
        *static_cast<size_t*>(p) = bytes;
        g_live_bytes += static_cast<int64_t>(bytes);
        p = static_cast<char*>(p) + sizeof(size_t);
    }
    *handle = p;
    // a view at a fixed distance from the host address, as a mapped pinned buffer may have
    *gpu_view = kind == tp::kResPinned ? static_cast<char*>(p) + (int64_t{1} << 40) : p;
    g_created[kind]++;
    return true;
}

void heap_destroy(int kind, int /*device*/, void* handle) {
    if (tp::is_buffer_kind(kind)) {
        handle = static_cast<char*>(handle) - sizeof(size_t);
        g_live_bytes -= static_cast<int64_t>(*static_cast<size_t*>(handle));
    }
    std::free(handle);
    g_destroyed[kind]++;
}

int heap_device() { return t_device; }

}  // namespace

extern "C" {

void* cache_emul_new() {
    return new tp::ResourceCache(tp::ResourceBackend{heap_create, heap_destroy, heap_device});
}
void cache_emul_delete(void* c) { delete static_cast<tp::ResourceCache*>(c); }
int cache_emul_acquire(void* c, int kind, int64_t bytes, void** handle) {
    return static_cast<tp::ResourceCache*>(c)->acquire(kind, bytes, handle);
}
int cache_emul_release(void* c, int kind, void* handle) {
    return static_cast<tp::ResourceCache*>(c)->release(kind, handle);
}
int64_t cache_emul_trim(void* c) { return static_cast<tp::ResourceCache*>(c)->trim(); }
void cache_emul_counts(void* c, int kind, int64_t out[6]) {
    const tp::ResourceCounts n = static_cast<tp::ResourceCache*>(c)->counts(kind);
    out[0] = n.hits;
    out[1] = n.misses;
    out[2] = n.idle;
    out[3] = n.leased;
    out[4] = n.idle_bytes;
    out[5] = n.leased_bytes;
}
// Returns 1 and fills kind / view offset from `ptr` / room if ptr is inside a leased buffer.
int cache_emul_find(void* c, const void* ptr, int* kind, int64_t* view_minus_ptr, int64_t* room) {
    const char* view = nullptr;
    if (!static_cast<tp::ResourceCache*>(c)->find_leased(ptr, kind, &view, room)) return 0;
    *view_minus_ptr = view - static_cast<const char*>(ptr);
    return 1;
}
int64_t cache_emul_capacity(int64_t bytes) { return tp::resource_capacity(bytes); }
void cache_emul_backend(int kind, int64_t out[3]) {
    out[0] = g_created[kind];
    out[1] = g_destroyed[kind];
    out[2] = g_live_bytes;
}
void cache_emul_fail_next(int n) { g_fail_next = n; }
void cache_emul_set_device(int d) { t_device = d; }

// `threads` x `rounds` acquire/release pairs of mixed sizes from concurrent threads; returns the
// number of anomalies seen (failed calls, a buffer handed to two holders at once).
int64_t cache_emul_hammer(void* c, int threads, int rounds) {
    tp::ResourceCache* cache = static_cast<tp::ResourceCache*>(c);
    std::atomic<int64_t> bad{0};
    std::vector<std::thread> pool;
    for (int t = 0; t < threads; ++t)
        pool.emplace_back([=, &bad] {
            uint64_t x = 0x9E3779B97F4A7C15ull * static_cast<uint64_t>(t + 1);
            for (int r = 0; r < rounds; ++r) {
                x = x * 6364136223846793005ull + 1442695040888963407ull;
                const int kind = static_cast<int>((x >> 60) & 3);
                const int64_t bytes = static_cast<int64_t>((x >> 20) % 100000);
                void* h = nullptr;
                if (cache->acquire(kind, bytes, &h) != 0 || !h) { bad++; continue; }
                if (tp::is_buffer_kind(kind)) {
                    // the holder's mark must survive until release: nobody else has this buffer
                    volatile uint64_t* mark = static_cast<uint64_t*>(h);
                    *mark = x;
                    std::this_thread::yield();
                    if (*mark != x) bad++;
                }
                if (cache->release(kind, h) != 0) bad++;
            }
        });
    for (auto& th : pool) th.join();
    return bad.load();
}

}  // extern "C"

// ---- BufferMap (buffer_map.hpp) over a made-up set of allocations ---------------------------------
#include "buffer_map.hpp"

namespace {

struct FakeMemory {
    int n = 0;
    const int64_t* lo = nullptr;
    const int64_t* hi = nullptr;
    const int* host = nullptr;
    bool bounds_known = true;
    int64_t queries = 0;
};
thread_local FakeMemory t_fake;

int fake_query(const void* p, tp::MemRange* r) {
    t_fake.queries++;
    const int64_t a = reinterpret_cast<intptr_t>(p);
    for (int i = 0; i < t_fake.n; ++i)
        if (t_fake.lo[i] <= a && a < t_fake.hi[i]) {
            r->lo = static_cast<uintptr_t>(t_fake.bounds_known ? t_fake.lo[i] : a);
            r->hi = static_cast<uintptr_t>(t_fake.bounds_known ? t_fake.hi[i] : a + 1);
            r->host = t_fake.host[i] != 0;
            r->view_delta = r->host ? (ptrdiff_t{1} << 40) : 0;
            return 0;
        }
    return 5;  // TP_ERR_BUFFER
}

}  // namespace

extern "C" {

// Runs `n_ops` locate() calls of one BufferMap against allocations [lo[i], hi[i]) (host[i]: mapped
// host memory).  status[k] and delta[k] (view minus address) are filled per call; returns the
// number of queries the map made.  checked == 0: a map without a query function.
int64_t bufmap_emul_run(int n_alloc, const int64_t* lo, const int64_t* hi, const int* host, int bounds_known,
                        int checked, int n_ops, const int64_t* addr, const int* allow_host, int* status,
                        int64_t* delta) {
    t_fake = FakeMemory{n_alloc, lo, hi, host, bounds_known != 0, 0};
    tp::BufferMap map(checked ? fake_query : nullptr);
    for (int k = 0; k < n_ops; ++k) {
        const char* p = reinterpret_cast<const char*>(static_cast<intptr_t>(addr[k]));
        const char* view = p;
        status[k] = map.locate(p, allow_host[k] != 0, &view);
        delta[k] = view - p;
    }
    return t_fake.queries;
}

}  // extern "C"
