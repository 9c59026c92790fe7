#include "model.hpp"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <sstream>

namespace tp {

bool ModelTable::valid() const {
    if (sizes.empty() || blocks.empty()) return false;
    for (size_t i = 1; i < sizes.size(); ++i)
        if (!(sizes[i] > sizes[i - 1])) return false;
    for (size_t i = 1; i < blocks.size(); ++i)
        if (!(blocks[i] > blocks[i - 1])) return false;
    if (!(sizes[0] > 0) || !(blocks[0] > 0)) return false;
    for (const auto& g : grid)
        if (g.size() != sizes.size() * blocks.size()) return false;
    for (const auto& c : copy)
        if (c.size() != sizes.size()) return false;
    return true;
}

namespace {

// Segment index i and weight w in [0, 1] so that x lies at (1-w)*axis[i] + w*axis[i+1]
// in log2 space; x is clamped to the axis range.  A one-point axis gives i = 0, w = 0.
void locate(const std::vector<double>& axis, double x, size_t* i, double* w) {
    if (axis.size() == 1 || x <= axis.front()) {
        *i = 0;
        *w = 0.0;
        return;
    }
    if (x >= axis.back()) {
        *i = axis.size() - 2;
        *w = 1.0;
        return;
    }
    size_t k = 0;
    while (x > axis[k + 1]) ++k;
    *i = k;
    *w = (std::log2(x) - std::log2(axis[k])) / (std::log2(axis[k + 1]) - std::log2(axis[k]));
}

}  // namespace

ModelTimes interpolate(const ModelTable& tb, double bytes, double block) {
    ModelTimes out;
    const double top = tb.sizes.back();
    const double scale = bytes > top ? bytes / top : 1.0;
    size_t si, bi;
    double sw, bw;
    locate(tb.sizes, std::min(bytes, top), &si, &sw);
    locate(tb.blocks, block, &bi, &bw);
    const size_t nb = tb.blocks.size();
    const size_t s1 = std::min(si + 1, tb.sizes.size() - 1), b1 = std::min(bi + 1, nb - 1);
    for (int p = 0; p < 4; ++p) {
        const std::vector<double>& g = tb.grid[p];
        const double lo = (1.0 - bw) * g[si * nb + bi] + bw * g[si * nb + b1];
        const double hi = (1.0 - bw) * g[s1 * nb + bi] + bw * g[s1 * nb + b1];
        out.t[p] = ((1.0 - sw) * lo + sw * hi) * scale;
    }
    for (int c = 0; c < 2; ++c) {
        const std::vector<double>& v = tb.copy[c];
        out.t[kD2H + c] = ((1.0 - sw) * v[si] + sw * v[s1]) * scale;
    }
    return out;
}

int select_method(const ModelTimes& m, double t_cpu_cpu, double t_gpu_gpu, double times[3]) {
    times[kMethodDevice] = m.t[kGpuPack] + t_gpu_gpu + m.t[kGpuUnpack];                                  // Eq. 1
    times[kMethodOneshot] = m.t[kHostPack] + t_cpu_cpu + m.t[kHostUnpack];                               // Eq. 2
    times[kMethodStaged] = m.t[kGpuPack] + m.t[kD2H] + t_cpu_cpu + m.t[kH2D] + m.t[kGpuUnpack];          // Eq. 3
    int best = kMethodDevice;
    for (int k = 1; k < 3; ++k)
        if (times[k] < times[best]) best = k;
    return best;
}

static const char* const kNames[kNumPrimitives] = {"gpu_pack", "gpu_unpack", "host_pack", "host_unpack", "d2h", "h2d"};

std::string serialize(const ModelTable& tb) {
    std::ostringstream os;
    os.precision(17);
    os << "tp_model 1\n";
    os << "sizes " << tb.sizes.size();
    for (double v : tb.sizes) os << ' ' << v;
    os << "\nblocks " << tb.blocks.size();
    for (double v : tb.blocks) os << ' ' << v;
    os << '\n';
    for (int p = 0; p < 4; ++p) {
        os << kNames[p];
        for (double v : tb.grid[p]) os << ' ' << v;
        os << '\n';
    }
    for (int c = 0; c < 2; ++c) {
        os << kNames[kD2H + c];
        for (double v : tb.copy[c]) os << ' ' << v;
        os << '\n';
    }
    return os.str();
}

bool parse(const std::string& text, ModelTable* out) {
    std::istringstream is(text);
    std::string word;
    int version = 0;
    if (!(is >> word >> version) || word != "tp_model" || version != 1) return false;
    ModelTable tb;
    size_t n = 0;
    if (!(is >> word >> n) || word != "sizes" || n == 0 || n > 4096) return false;
    tb.sizes.resize(n);
    for (double& v : tb.sizes)
        if (!(is >> v)) return false;
    if (!(is >> word >> n) || word != "blocks" || n == 0 || n > 4096) return false;
    tb.blocks.resize(n);
    for (double& v : tb.blocks)
        if (!(is >> v)) return false;
    for (int p = 0; p < kNumPrimitives; ++p) {
        if (!(is >> word) || word != kNames[p]) return false;
        std::vector<double>& dst = p < 4 ? tb.grid[p] : tb.copy[p - 4];
        dst.resize(p < 4 ? tb.sizes.size() * tb.blocks.size() : tb.sizes.size());
        for (double& v : dst)
            if (!(is >> v) || !(v >= 0.0)) return false;
    }
    if (!tb.valid()) return false;
    *out = std::move(tb);
    return true;
}

Model& Model::instance() {
    static Model m;
    return m;
}

void Model::set(ModelTable table) {
    std::lock_guard<std::mutex> lock(mu_);
    table_ = std::move(table);
    loaded_ = true;
    memo_.clear();
}

bool Model::loaded() const {
    std::lock_guard<std::mutex> lock(mu_);
    return loaded_;
}

ModelTable Model::table() const {
    std::lock_guard<std::mutex> lock(mu_);
    return table_;
}

bool Model::query(int64_t bytes, int64_t block, ModelTimes* out) {
    std::lock_guard<std::mutex> lock(mu_);
    if (!loaded_) return false;
    const Key key{bytes, block};
    auto it = memo_.find(key);
    if (it == memo_.end()) {
        if (memo_.size() > (1u << 16)) memo_.clear();
        it = memo_.emplace(key, interpolate(table_, static_cast<double>(bytes), static_cast<double>(block))).first;
    }
    *out = it->second;
    return true;
}

}  // namespace tp
