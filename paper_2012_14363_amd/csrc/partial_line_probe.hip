// Stand-alone measurement of the hardware property the staged unpack rests on: the rate at which
// partially written memory lines retire, against the spacing of the lines written at one time,
// the source of the stored bytes (resident in L2 or streamed from HBM), the store's cache policy
// and the number of workgroups.  One byte per row, one row per thread and loop trip, rows `pitch`
// bytes apart; every store lands in a line of its own (pitch >= 128) or shares it (pitch 64).
// Not part of the library; prints one table.  Usage: partial_line_probe [log2 of rows, 20..23]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                              \
        }                                                                              \
    } while (0)

namespace {

constexpr int kThreads = 256;
constexpr size_t kResident = size_t{1} << 20;  // bytes of source that are reused when it is to stay in L2

// Workgroup g takes tiles g, g + gridDim.x, ... of 256 rows.  Rows first, first + step, ... (`count` of
// them) of the typed buffer; the byte stored into row r comes from src[r & mask].
template <bool THROUGH>
__global__ void __launch_bounds__(kThreads) scatter(const uint8_t* src, size_t mask, uint8_t* typed, size_t first,
                                                    size_t step, size_t count, size_t pitch) {
    const size_t tiles = (count + kThreads - 1) / kThreads;
    for (size_t t = blockIdx.x; t < tiles; t += gridDim.x) {
        const size_t i = t * kThreads + threadIdx.x;
        if (i >= count) break;
        const size_t r = first + i * step;
        const uint32_t v = src[r & mask];
        uint8_t* p = typed + r * pitch;
        if (THROUGH) asm volatile("global_store_byte %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
        else asm volatile("global_store_byte %0, %1, off nt" : : "v"(p), "v"(v) : "memory");
    }
}

struct Setup {
    uint8_t* typed = nullptr;
    size_t typed_bytes = 0;
    uint8_t* source = nullptr;  // `windows` windows of `rows` bytes
    size_t rows = 0, windows = 0;
    hipEvent_t a{}, b{};
};

// Best of four timings, in G rows/s.  `resident`: every repetition reads the same first MiB of the
// source; otherwise repetition k reads window k (never the same within 512 MiB of reads).
double rate(Setup& s, size_t pitch, int passes, int grid, bool through, bool resident, size_t* window) {
    if ((s.rows - 1) * pitch + 1 > s.typed_bytes || s.rows % (static_cast<size_t>(kThreads) * passes) != 0) {
        std::printf("bad shape\n");
        std::exit(2);
    }
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {
        const uint8_t* src = resident ? s.source : s.source + (*window)++ % s.windows * s.rows;
        const size_t mask = resident ? kResident - 1 : s.rows - 1;   // rows is a power of two
        CK(hipEventRecord(s.a));
        for (int p = 0; p < passes; ++p) {
            if (through) hipLaunchKernelGGL(scatter<true>, dim3(grid), dim3(kThreads), 0, 0, src, mask, s.typed, p, passes, s.rows / passes, pitch);
            else hipLaunchKernelGGL(scatter<false>, dim3(grid), dim3(kThreads), 0, 0, src, mask, s.typed, p, passes, s.rows / passes, pitch);
        }
        CK(hipEventRecord(s.b));
        CK(hipEventSynchronize(s.b));
        float ms = 0;
        CK(hipEventElapsedTime(&ms, s.a, s.b));
        if (ms < best) best = ms;
    }
    CK(hipGetLastError());
    return static_cast<double>(s.rows) / (best * 1e-3) / 1e9;
}

}  // namespace

int main(int argc, char** argv) {
    const int lg = argc > 1 ? std::atoi(argv[1]) : 22;
    if (lg < 20 || lg > 23) {
        std::printf("usage: partial_line_probe [log2 of rows, 20..23]\n");
        return 2;
    }
    Setup s;
    s.rows = size_t{1} << lg;
    s.typed_bytes = s.rows * 4096;
    s.windows = (size_t{1} << 29) / s.rows;   // 512 MiB of source windows
    CK(hipMalloc(&s.typed, s.typed_bytes));
    CK(hipMalloc(&s.source, s.windows * s.rows));
    CK(hipMemset(s.typed, 1, s.typed_bytes));
    CK(hipMemset(s.source, 2, s.windows * s.rows));
    CK(hipEventCreate(&s.a));
    CK(hipEventCreate(&s.b));
    size_t window = 0;
    std::printf("one-byte rows, 2^%d of them, one store per thread and loop trip; G rows/s, best of 4\n\n", lg);
    std::printf("| pitch | sc1 nt, source in L2, 256 workgroups | same, source from HBM | nt, source in L2 | sc1 nt, source in L2, in 512/pitch passes |\n");
    std::printf("|---|---|---|---|---|\n");
    for (size_t pitch : {64, 128, 192, 256, 320, 384, 448, 512, 576, 640, 768, 1024, 1536, 2048, 4096}) {
        const double r1 = rate(s, pitch, 1, 256, true, true, &window);
        const double r2 = rate(s, pitch, 1, 256, true, false, &window);
        const double r3 = rate(s, pitch, 1, 256, false, true, &window);
        std::printf("| %zu | %.1f | %.1f | %.1f |", pitch, r1, r2, r3);
        if (pitch == 128 || pitch == 256) std::printf(" %.1f |\n", rate(s, pitch, static_cast<int>(512 / pitch), 256, true, true, &window));
        else std::printf(" |\n");
        std::fflush(stdout);
    }
    std::printf("\n| workgroups at 512-byte pitch (sc1 nt, source in L2) | G rows/s |\n|---|---|\n");
    for (int grid : {64, 128, 256, 512, 1024, 4096}) {
        std::printf("| %d | %.1f |\n", grid, rate(s, 512, 1, grid, true, true, &window));
        std::fflush(stdout);
    }
    CK(hipDeviceSynchronize());
    CK(hipFree(s.typed));
    CK(hipFree(s.source));
    return 0;
}
