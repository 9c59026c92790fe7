// Cache of the runtime resources a send/receive layer asks for again and again: device buffers,
// pinned host buffers, streams and events (paper Sec. 5: repeated requests are served from a
// cache in tens to hundreds of nanoseconds instead of the microseconds to milliseconds the
// runtime takes to create them).
//
// A resource is leased (`acquire`), used by one caller, and given back (`release`); released
// resources stay alive in idle lists, keyed by device and, for buffers, by a size class, and the
// next request of that class takes one instead of calling the runtime.  Nothing is destroyed
// before `trim`.  The class is independent of HIP: creation and destruction go through a
// ResourceBackend, so the bookkeeping can be tested on the host heap.
#pragma once

#include <atomic>
#include <cstddef>
#include <cstdint>
#include <map>
#include <mutex>
#include <vector>

namespace tp {

enum ResourceKind : int { kResDevice = 0, kResPinned = 1, kResStream = 2, kResEvent = 3, kResKinds = 4 };

inline bool is_buffer_kind(int kind) { return kind == kResDevice || kind == kResPinned; }

struct ResourceBackend {
    // Makes a resource on `device`.  *handle is what the caller uses (a buffer's address, a
    // hipStream_t, a hipEvent_t); for buffers *gpu_view is the address kernels use for it.
    bool (*create)(int kind, int device, size_t bytes, void** handle, void** gpu_view);
    void (*destroy)(int kind, int device, void* handle);
    int (*current_device)();  // negative on failure
};

struct ResourceCounts {
    int64_t hits = 0;    // acquires served from an idle list
    int64_t misses = 0;  // acquires that created a resource
    int64_t idle = 0;    // resources alive and not leased
    int64_t leased = 0;
    int64_t idle_bytes = 0;  // buffers only: capacities, not requested sizes
    int64_t leased_bytes = 0;
};

// Capacity (bytes) a buffer request is rounded up to: four classes per power of two, 4 KiB at
// least, so a buffer is at most 25 % larger than asked for.  Returns 0 if `bytes` is negative
// or too large to round.
int64_t resource_capacity(int64_t bytes);

class ResourceCache {
public:
    explicit ResourceCache(ResourceBackend backend);
    ~ResourceCache();  // destroys idle resources; leased ones are the holders' to give back first
    ResourceCache(const ResourceCache&) = delete;
    ResourceCache& operator=(const ResourceCache&) = delete;

    // Leases a resource of the calling thread's current device.  `bytes` is the least capacity of
    // a buffer (0 is allowed) and ignored for streams and events.  Returns a TP_* status.
    int acquire(int kind, int64_t bytes, void** handle);
    // Gives a lease back.  The caller must have waited for all work that uses the resource.
    // kErrArg if `handle` is not a current lease of that kind.
    int release(int kind, void* handle);
    // Destroys every idle resource (all devices); returns the buffer bytes freed.
    int64_t trim();
    ResourceCounts counts(int kind) const;

    // True if `ptr` lies inside a buffer leased from here.  *kind is the buffer's kind, *gpu_view
    // the address of that byte as kernels see it, *room the bytes from `ptr` to the buffer's end.
    bool find_leased(const void* ptr, int* kind, const char** gpu_view, int64_t* room) const;

private:
    struct Item {
        void* handle = nullptr;
        char* gpu_view = nullptr;
        int64_t capacity = 0;
        int device = 0;
        int kind = 0;
    };
    struct IdleKey {
        int device, kind;
        int64_t capacity;
        bool operator<(const IdleKey& o) const {
            if (device != o.device) return device < o.device;
            if (kind != o.kind) return kind < o.kind;
            return capacity < o.capacity;
        }
    };
    void destroy_idle_locked(int64_t* bytes);

    ResourceBackend backend_;
    mutable std::mutex mu_;
    std::map<IdleKey, std::vector<Item>> idle_;
    std::map<uintptr_t, Item> leased_[kResKinds];  // by handle address
    ResourceCounts counts_[kResKinds];
    std::atomic<int64_t> leased_buffers_{0};  // lets find_leased skip the lock when nothing is out
};

// The library's own cache, backed by HIP.  Never destroyed: the runtime may already be gone when
// static destructors run.
ResourceCache& library_resources();

}  // namespace tp
