// A small program for the thread sanitizer (tests/test_sanitized_builds_cpu.py builds it with
// -fsanitize=thread and runs it): the threaded paths of the host-side code without an interpreter in
// the process - the handle table and commit under eight threads, the resource cache under eight
// threads, and the C oracle's threaded copy against its single-threaded one.  Tests only.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

extern "C" {
int64_t types_emul_hammer(int threads, int rounds);
void* cache_emul_new();
void cache_emul_delete(void*);
int64_t cache_emul_hammer(void*, int threads, int rounds);
int64_t cache_emul_trim(void*);
int64_t tmo_copy(int direction, const int64_t* enc, int64_t n, uint8_t* typed, int64_t typed_len, int64_t origin,
                 int64_t count, uint8_t* packed, int64_t packed_len, int64_t position, int nthreads);
}

int main() {
    int64_t bad = types_emul_hammer(8, 2000);
    std::printf("handle table and commit: %lld wrong\n", static_cast<long long>(bad));

    void* cache = cache_emul_new();
    int64_t c = cache_emul_hammer(cache, 8, 3000);
    cache_emul_trim(cache);
    c += cache_emul_hammer(cache, 8, 3000);
    cache_emul_delete(cache);
    std::printf("resource cache: %lld wrong\n", static_cast<long long>(c));
    bad += c;

    // vector(5000, 3, 7, BYTE), 4 objects: kind 2 = vector (count, blocklength, stride), kind 0 = named (size)
    const int64_t enc[] = {2, 5000, 3, 7, 0, 1};
    const int64_t extent = (5000 - 1) * 7 + 3, size = 5000 * 3, objects = 4;
    std::vector<uint8_t> typed(static_cast<size_t>(extent * objects)), one(static_cast<size_t>(size * objects)), many(one.size());
    for (size_t i = 0; i < typed.size(); ++i) typed[i] = static_cast<uint8_t>(i * 131 + 7);
    const int64_t p1 = tmo_copy(0, enc, 6, typed.data(), static_cast<int64_t>(typed.size()), 0, objects, one.data(),
                                static_cast<int64_t>(one.size()), 0, 1);
    const int64_t p8 = tmo_copy(0, enc, 6, typed.data(), static_cast<int64_t>(typed.size()), 0, objects, many.data(),
                                static_cast<int64_t>(many.size()), 0, 8);
    const bool same = p1 == size * objects && p8 == p1 && std::memcmp(one.data(), many.data(), one.size()) == 0;
    std::printf("threaded oracle copy: %s\n", same ? "equal" : "DIFFERENT");
    bad += same ? 0 : 1;
    return bad == 0 ? 0 : 1;
}
