#include "resource_cache.hpp"

#include "status.hpp"

namespace tp {

int64_t resource_capacity(int64_t bytes) {
    constexpr int64_t kMin = 4096;
    if (bytes < 0) return 0;
    if (bytes <= kMin) return kMin;
    if (bytes > (int64_t{1} << 61)) return 0;
    // quarter steps of the power of two below `bytes`
    const int top = 63 - __builtin_clzll(static_cast<uint64_t>(bytes));
    const int64_t step = int64_t{1} << (top - 2);
    return (bytes + step - 1) / step * step;
}

ResourceCache::ResourceCache(ResourceBackend backend) : backend_(backend) {}

ResourceCache::~ResourceCache() { trim(); }

int ResourceCache::acquire(int kind, int64_t bytes, void** handle) {
    if (!handle || kind < 0 || kind >= kResKinds) return kErrArg;
    int64_t capacity = 0;
    if (is_buffer_kind(kind)) {
        if (bytes < 0) return kErrArg;
        capacity = resource_capacity(bytes);
        if (capacity == 0) return kErrRange;
    }
    const int device = backend_.current_device();
    if (device < 0) return kErrOther;

    Item item;
    bool hit = false;
    {
        std::lock_guard<std::mutex> lock(mu_);
        auto it = idle_.find(IdleKey{device, kind, capacity});
        if (it != idle_.end() && !it->second.empty()) {
            item = it->second.back();
            it->second.pop_back();
            hit = true;
            counts_[kind].idle -= 1;
            counts_[kind].idle_bytes -= item.capacity;
        }
    }
    if (!hit) {
        // created outside the lock: the runtime may take milliseconds
        item.device = device;
        item.kind = kind;
        item.capacity = capacity;
        void* view = nullptr;
        bool ok = backend_.create(kind, device, static_cast<size_t>(capacity), &item.handle, &view);
        if (!ok) {
            // out of memory, perhaps because of what sits idle here: give that back and retry once
            trim();
            ok = backend_.create(kind, device, static_cast<size_t>(capacity), &item.handle, &view);
        }
        if (!ok || !item.handle) return kErrOther;
        item.gpu_view = static_cast<char*>(view);
    }
    {
        std::lock_guard<std::mutex> lock(mu_);
        leased_[kind][reinterpret_cast<uintptr_t>(item.handle)] = item;
        ResourceCounts& c = counts_[kind];
        (hit ? c.hits : c.misses) += 1;
        c.leased += 1;
        c.leased_bytes += item.capacity;
        if (is_buffer_kind(kind)) leased_buffers_.fetch_add(1, std::memory_order_release);
    }
    *handle = item.handle;
    return kSuccess;
}

int ResourceCache::release(int kind, void* handle) {
    if (!handle || kind < 0 || kind >= kResKinds) return kErrArg;
    std::lock_guard<std::mutex> lock(mu_);
    auto it = leased_[kind].find(reinterpret_cast<uintptr_t>(handle));
    if (it == leased_[kind].end()) return kErrArg;
    const Item item = it->second;
    leased_[kind].erase(it);
    if (is_buffer_kind(kind)) leased_buffers_.fetch_sub(1, std::memory_order_release);
    ResourceCounts& c = counts_[kind];
    c.leased -= 1;
    c.leased_bytes -= item.capacity;
    c.idle += 1;
    c.idle_bytes += item.capacity;
    idle_[IdleKey{item.device, kind, item.capacity}].push_back(item);
    return kSuccess;
}

void ResourceCache::destroy_idle_locked(int64_t* bytes) {
    for (auto& entry : idle_) {
        for (const Item& item : entry.second) {
            backend_.destroy(item.kind, item.device, item.handle);
            counts_[item.kind].idle -= 1;
            counts_[item.kind].idle_bytes -= item.capacity;
            *bytes += item.capacity;
        }
    }
    idle_.clear();
}

int64_t ResourceCache::trim() {
    int64_t bytes = 0;
    std::lock_guard<std::mutex> lock(mu_);
    destroy_idle_locked(&bytes);
    return bytes;
}

ResourceCounts ResourceCache::counts(int kind) const {
    if (kind < 0 || kind >= kResKinds) return ResourceCounts();
    std::lock_guard<std::mutex> lock(mu_);
    return counts_[kind];
}

bool ResourceCache::find_leased(const void* ptr, int* kind, const char** gpu_view, int64_t* room) const {
    if (leased_buffers_.load(std::memory_order_acquire) == 0) return false;
    const uintptr_t p = reinterpret_cast<uintptr_t>(ptr);
    std::lock_guard<std::mutex> lock(mu_);
    for (int k : {int(kResDevice), int(kResPinned)}) {
        auto it = leased_[k].upper_bound(p);
        if (it == leased_[k].begin()) continue;
        --it;
        const Item& item = it->second;
        const uintptr_t base = it->first;
        if (p - base >= static_cast<uint64_t>(item.capacity)) continue;
        *kind = k;
        *gpu_view = item.gpu_view + (p - base);
        *room = item.capacity - static_cast<int64_t>(p - base);
        return true;
    }
    return false;
}

}  // namespace tp
