// Measured performance model for choosing how packed data reaches the host
// (paper Sec. 4, Eq. 1-3, and Sec. 6.3: sparse system measurements, interpolated
// at run time, results memoised).
#pragma once

#include <cstdint>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

namespace tp {

// The six primitives that can be measured on one GPU (seconds per operation).
enum Primitive : int { kGpuPack = 0, kGpuUnpack, kHostPack, kHostUnpack, kD2H, kH2D, kNumPrimitives };

struct ModelTimes {
    double t[kNumPrimitives] = {};
};

// A sparse table: pack/unpack times over (object bytes, contiguous block bytes),
// copy times over object bytes.  Sizes and blocks are strictly increasing.
struct ModelTable {
    std::vector<double> sizes;   // object bytes
    std::vector<double> blocks;  // contiguous block length, bytes
    std::vector<double> grid[4];  // kGpuPack..kHostUnpack: sizes.size() * blocks.size(), size-major
    std::vector<double> copy[2];  // kD2H, kH2D: sizes.size()
    bool valid() const;
};

// Interpolates `table` at (bytes, block): bilinear in (log2 bytes, log2 block),
// block clamped to the measured range, bytes below the range clamped (latency
// floor), above it scaled proportionally from the largest measured size
// (bandwidth regime).
ModelTimes interpolate(const ModelTable& table, double bytes, double block);

enum Method : int { kMethodDevice = 0, kMethodOneshot = 1, kMethodStaged = 2 };

// Eq. 1-3 with the two transport terms that need a second rank supplied by the caller.
// times[m] receives T_device, T_oneshot, T_staged; returns the fastest method.
int select_method(const ModelTimes& m, double t_cpu_cpu, double t_gpu_gpu, double times[3]);

std::string serialize(const ModelTable& table);
bool parse(const std::string& text, ModelTable* table);

// The process-wide model: a table plus a memo of interpolated queries.
class Model {
public:
    static Model& instance();
    void set(ModelTable table);
    bool loaded() const;
    ModelTable table() const;
    // Memoised interpolate(); false if no table is loaded.
    bool query(int64_t bytes, int64_t block, ModelTimes* out);

private:
    mutable std::mutex mu_;
    ModelTable table_;
    bool loaded_ = false;
    struct Key {
        int64_t bytes, block;
        bool operator==(const Key& o) const { return bytes == o.bytes && block == o.block; }
    };
    struct KeyHash {
        size_t operator()(const Key& k) const {
            return std::hash<int64_t>()(k.bytes * 1000003 + k.block);
        }
    };
    std::unordered_map<Key, ModelTimes, KeyHash> memo_;
};

}  // namespace tp
