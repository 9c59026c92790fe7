/*
 * pack_selftest: the pack/unpack path driven from plain C through include/tp_pack.h alone - no
 * HIP headers, no Python.  Buffers come from the library's resource cache; data reaches the
 * device and comes back through the zero-copy form of the calls themselves (the contiguous side
 * in pinned host memory, paper Sec. 4).
 *
 * For a 3D block of a 3D byte array (paper Sec. 2, the cuboid built as hvector of hvector of
 * contiguous) it uploads a pattern, packs the block on the GPU, and compares with three nested
 * loops over the same array on the CPU; then unpacks into a poisoned device array and checks
 * that exactly the block changed.  Exit status 0 and "ok" on success.  Needs a GPU.
 * Usage: pack_selftest [a0 a1 a2]   (block extents in bytes / rows / planes; array is 64 x 48 x 40)
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "tp_pack.h"

enum { E0 = 64, E1 = 48, E2 = 40 };

static void check(int rc, const char *what) {
    if (rc != TP_SUCCESS) {
        fprintf(stderr, "%s: tp error %d: %s\n", what, rc, tp_error_string(rc));
        exit(1);
    }
}

static unsigned char pattern(int64_t i) { return (unsigned char)((i * 2654435761u) >> 13); }

int main(int argc, char **argv) {
    int a0 = argc > 3 ? atoi(argv[1]) : 13, a1 = argc > 3 ? atoi(argv[2]) : 17, a2 = argc > 3 ? atoi(argv[3]) : 9;
    if (a0 < 1 || a0 > E0 || a1 < 1 || a1 > E1 || a2 < 1 || a2 > E2) {
        fprintf(stderr, "block must fit the %d x %d x %d array\n", E0, E1, E2);
        return 2;
    }
    const int64_t total = (int64_t)E0 * E1 * E2, packed = (int64_t)a0 * a1 * a2;

    tp_type row, plane, block, whole;
    check(tp_type_contiguous(a0, TP_BYTE, &row), "contiguous");
    check(tp_type_create_hvector(a1, 1, E0, row, &plane), "hvector");
    check(tp_type_create_hvector(a2, 1, (int64_t)E0 * E1, plane, &block), "hvector");
    check(tp_type_contiguous((int)total, TP_BYTE, &whole), "contiguous");
    check(tp_type_commit(&block), "commit");
    check(tp_type_commit(&whole), "commit");
    tp_type_free(&row);
    tp_type_free(&plane);

    void *array_dev, *poisoned_dev, *host, *stream;
    check(tp_resource_acquire(TP_RES_DEVICE, total, &array_dev), "device buffer");
    check(tp_resource_acquire(TP_RES_DEVICE, total, &poisoned_dev), "device buffer");
    check(tp_resource_acquire(TP_RES_PINNED, 2 * total + 64, &host), "pinned buffer");
    check(tp_resource_acquire(TP_RES_STREAM, 0, &stream), "stream");
    unsigned char *h = host, *out = h + total;

    /* upload: unpack the pinned pattern into the device array as one contiguous run */
    for (int64_t i = 0; i < total; ++i) h[i] = pattern(i);
    int64_t pos = 0;
    check(tp_unpack(h, total, &pos, array_dev, 1, whole, stream), "upload");

    /* pack the block on the GPU straight into pinned memory, behind a 5-byte prefix */
    memset(out, 0xEE, (size_t)total + 64);
    pos = 5;
    check(tp_pack(array_dev, 1, block, out, packed + 5, &pos, stream), "pack");
    int bad = pos != packed + 5;
    int64_t k = 5;
    for (int z = 0; z < a2; ++z)
        for (int y = 0; y < a1; ++y)
            for (int x = 0; x < a0; ++x) bad += out[k++] != pattern(((int64_t)z * E1 + y) * E0 + x);
    for (int i = 0; i < 5; ++i) bad += out[i] != 0xEE;
    bad += out[k] != 0xEE;

    /* unpack the packed block into an array of 0xA5, download it, and look at every byte */
    memset(h, 0xA5, (size_t)total);
    pos = 0;
    check(tp_unpack(h, total, &pos, poisoned_dev, 1, whole, stream), "poison");
    pos = 5;
    check(tp_unpack(out, packed + 5, &pos, poisoned_dev, 1, block, stream), "unpack");
    pos = 0;
    check(tp_pack(poisoned_dev, 1, whole, h, total, &pos, stream), "download");
    for (int z = 0; z < E2; ++z)
        for (int y = 0; y < E1; ++y)
            for (int x = 0; x < E0; ++x) {
                const int64_t i = ((int64_t)z * E1 + y) * E0 + x;
                const int inside = x < a0 && y < a1 && z < a2;
                bad += h[i] != (inside ? pattern(i) : 0xA5);
            }

    check(tp_resource_release(TP_RES_STREAM, stream), "release");
    check(tp_resource_release(TP_RES_PINNED, host), "release");
    check(tp_resource_release(TP_RES_DEVICE, poisoned_dev), "release");
    check(tp_resource_release(TP_RES_DEVICE, array_dev), "release");
    check(tp_resource_trim(NULL), "trim");
    tp_type_free(&block);
    tp_type_free(&whole);
    if (bad) {
        printf("FAILED: %d mismatching bytes (block %d x %d x %d)\n", bad, a0, a1, a2);
        return 1;
    }
    printf("ok: block %d x %d x %d of %d x %d x %d, %lld bytes packed and unpacked\n", a0, a1, a2, E0, E1, E2,
           (long long)packed);
    return 0;
}
