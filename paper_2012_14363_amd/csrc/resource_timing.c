/*
 * resource_timing: what the resource cache saves (paper Sec. 5 states the aim: repeated requests
 * served in tens to hundreds of nanoseconds instead of the runtime's microseconds to
 * milliseconds).
 *
 * For each kind - device buffer, pinned host buffer, stream, event - it takes `misses` leases
 * without giving any back, so each one is created by the runtime (the median is the creation
 * cost), releases them, and then times `pairs` acquire/release pairs, all of which the cache
 * serves.  Buffers are 1 MiB.  Needs a GPU.  Plain C, through the C ABI only.
 * Output: one JSON array on stdout.  Usage: resource_timing [pairs [misses]]
 */
#define _POSIX_C_SOURCE 199309L
#include <stdio.h>
#include <stdlib.h>
#include <time.h>

#include "tp_pack.h"

static double now_ns(void) {
    struct timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return 1e9 * (double)ts.tv_sec + (double)ts.tv_nsec;
}

static int cmp_double(const void *a, const void *b) {
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

static void check(int rc) {
    if (rc != TP_SUCCESS) { fprintf(stderr, "tp error %d: %s\n", rc, tp_error_string(rc)); exit(1); }
}

int main(int argc, char **argv) {
    int pairs = argc > 1 ? atoi(argv[1]) : 1000000;
    int misses = argc > 2 ? atoi(argv[2]) : 16;
    if (pairs < 1) pairs = 1;
    if (misses < 1) misses = 1;
    if (misses > 256) misses = 256;
    static const char *names[4] = {"device buffer", "pinned host buffer", "stream", "event"};
    const int64_t bytes = 1 << 20;
    void *held[256];
    double t_miss[256];
    printf("[");
    for (int kind = 0; kind < 4; ++kind) {
        for (int i = 0; i < misses; ++i) {
            double t0 = now_ns();
            check(tp_resource_acquire(kind, bytes, &held[i]));
            t_miss[i] = now_ns() - t0;
        }
        for (int i = 0; i < misses; ++i) check(tp_resource_release(kind, held[i]));
        qsort(t_miss, (size_t)misses, sizeof(double), cmp_double);
        void *h = NULL;
        double t0 = now_ns();
        for (int i = 0; i < pairs; ++i) {
            check(tp_resource_acquire(kind, bytes, &h));
            check(tp_resource_release(kind, h));
        }
        double per_pair = (now_ns() - t0) / pairs;
        tp_resource_counts c;
        check(tp_resource_stats(kind, &c));
        printf("%s{\"kind\": \"%s\", \"create_median_ns\": %.0f, \"create_min_ns\": %.0f, \"creations\": %d, "
               "\"cached_pair_ns\": %.1f, \"pairs\": %d, \"hits\": %lld, \"misses\": %lld}",
               kind ? ", " : "", names[kind], t_miss[misses / 2], t_miss[0], misses, per_pair, pairs,
               (long long)c.hits, (long long)c.misses);
    }
    printf("]\n");
    check(tp_resource_trim(NULL));
    return 0;
}
