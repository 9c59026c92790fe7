/*
 * commit_timing: time datatype construction and commit through the C ABI.
 *
 * Mirrors the measurement of the paper's Sec. 6.1 (commit figure): for a set of 3D
 * objects described in four families - subarray; hvector of vector; hvector of
 * hvector of vector; subarray of vector - run many create / commit / free cycles
 * and report the trimean (Q1 + 2*median + Q3)/4 of each phase.  The paper's own 15
 * parameter sets exist only in its figure; the shapes here stand in (the same ones
 * workloads/configs.py lists), plus the five benchmark datatypes.
 *
 * With a model file (written by tp_model_save) it also times the memoised
 * performance-model query, tp_model_select, the overhead the paper reports in
 * Sec. 6.3 for its own model.
 *
 * Plain C on purpose: it also proves include/tp_pack.h is usable from C.
 * Output: one JSON array on stdout.  Usage: commit_timing [iterations [model_file]]
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

static double trimean(double *v, int n) {
    qsort(v, (size_t)n, sizeof(double), cmp_double);
    return (v[n / 4] + 2.0 * v[n / 2] + v[3 * n / 4]) / 4.0;
}

typedef struct Shape { int a0, a1, a2, e0, e1, e2; } Shape;

/* Each builder returns the uncommitted top-level type and frees its intermediates. */
typedef tp_type (*Builder)(const Shape *);

static void check(int rc) {
    if (rc != TP_SUCCESS) { fprintf(stderr, "tp error %d: %s\n", rc, tp_error_string(rc)); exit(1); }
}

static tp_type b_subarray(const Shape *s) {
    int sizes[3] = {s->a2, s->a1, s->a0}, subs[3] = {s->e2, s->e1, s->e0}, starts[3] = {0, 0, 0};
    tp_type t;
    check(tp_type_create_subarray(3, sizes, subs, starts, TP_ORDER_C, TP_BYTE, &t));
    return t;
}

static tp_type b_hvector_vector(const Shape *s) {
    tp_type plane, t;
    check(tp_type_vector(s->e1, s->e0, s->a0, TP_BYTE, &plane));
    check(tp_type_create_hvector(s->e2, 1, (int64_t)s->a0 * s->a1, plane, &t));
    tp_type_free(&plane);
    return t;
}

static tp_type b_hvector_hvector_vector(const Shape *s) {
    tp_type row, plane, t;
    check(tp_type_vector(1, s->e0, 1, TP_BYTE, &row));
    check(tp_type_create_hvector(s->e1, 1, s->a0, row, &plane));
    check(tp_type_create_hvector(s->e2, 1, (int64_t)s->a0 * s->a1, plane, &t));
    tp_type_free(&row);
    tp_type_free(&plane);
    return t;
}

static tp_type b_hvector_hvector_vector4(const Shape *s) {
    tp_type row, plane, t;
    check(tp_type_vector(s->e0 / 4, 4, 4, TP_BYTE, &row));
    check(tp_type_create_hvector(s->e1, 1, s->a0, row, &plane));
    check(tp_type_create_hvector(s->e2, 1, (int64_t)s->a0 * s->a1, plane, &t));
    tp_type_free(&row);
    tp_type_free(&plane);
    return t;
}

static tp_type b_subarray_vector(const Shape *s) {
    tp_type plane, t;
    int sizes[1] = {s->a2}, subs[1] = {s->e2}, starts[1] = {0};
    check(tp_type_vector(s->e1, s->e0, s->a0, TP_BYTE, &plane));
    check(tp_type_create_subarray(1, sizes, subs, starts, TP_ORDER_C, plane, &t));
    tp_type_free(&plane);
    return t;
}

/* the five benchmark datatypes (shape argument unused) */
static tp_type b_cfg_vector(const Shape *s) {
    (void)s;
    tp_type t;
    check(tp_type_vector(64, 8, 512, TP_BYTE, &t));
    return t;
}

static tp_type b_cfg_block3d(const Shape *s) {
    (void)s;
    tp_type row, plane, t;
    check(tp_type_contiguous(16, TP_BYTE, &row));
    check(tp_type_create_hvector(256, 1, 512, row, &plane));
    check(tp_type_create_hvector(256, 1, 512 * 512, plane, &t));
    tp_type_free(&row);
    tp_type_free(&plane);
    return t;
}

static tp_type b_cfg_halo_face(const Shape *s) {
    (void)s;
    int sizes[3] = {512, 512, 512}, subs[3] = {506, 506, 3}, starts[3] = {3, 3, 3};
    tp_type t;
    check(tp_type_create_subarray(3, sizes, subs, starts, TP_ORDER_C, TP_DOUBLE, &t));
    return t;
}

static tp_type b_cfg_tiny_runs(const Shape *s) {
    (void)s;
    tp_type t;
    check(tp_type_vector(1 << 24, 3, 64, TP_BYTE, &t));
    return t;
}

static tp_type b_cfg_nested(const Shape *s) {
    (void)s;
    int sizes[3] = {64, 64, 64}, subs[3] = {8, 16, 64}, starts[3] = {3, 5, 0};
    tp_type sub, hv, t;
    check(tp_type_create_subarray(3, sizes, subs, starts, TP_ORDER_C, TP_FLOAT, &sub));
    check(tp_type_create_hvector(16, 1, 8192, sub, &hv));
    check(tp_type_vector(4, 1, 2, hv, &t));
    tp_type_free(&sub);
    tp_type_free(&hv);
    return t;
}

int main(int argc, char **argv) {
    int iters = argc > 1 ? atoi(argv[1]) : 30000;
    if (iters < 8) iters = 8;
    static const Shape shapes[3] = {{256, 512, 1024, 100, 13, 47}, {512, 512, 512, 64, 64, 64}, {512, 512, 512, 512, 16, 16}};
    struct { const char *name; Builder build; int per_shape; } cases[] = {
        {"subarray", b_subarray, 1},
        {"hvector(vector)", b_hvector_vector, 1},
        {"hvector(hvector(vector(1,e0,1)))", b_hvector_hvector_vector, 1},
        {"hvector(hvector(vector(e0/4,4,4)))", b_hvector_hvector_vector4, 1},
        {"subarray(vector)", b_subarray_vector, 1},
        {"workload: 2D vector 64x8 @512", b_cfg_vector, 0},
        {"workload: 3D block 16x256x256", b_cfg_block3d, 0},
        {"workload: halo x-face subarray", b_cfg_halo_face, 0},
        {"workload: 2^24 runs of 3 B", b_cfg_tiny_runs, 0},
        {"workload: nested 4-level", b_cfg_nested, 0},
    };
    double *t_create = malloc(sizeof(double) * (size_t)iters), *t_commit = malloc(sizeof(double) * (size_t)iters);
    if (!t_create || !t_commit) return 1;
    printf("[");
    int first = 1;
    for (size_t c = 0; c < sizeof cases / sizeof cases[0]; ++c) {
        for (int s = 0; s < (cases[c].per_shape ? 3 : 1); ++s) {
            int ndims = 0;
            for (int i = 0; i < iters; ++i) {
                double t0 = now_ns();
                tp_type t = cases[c].build(&shapes[s]);
                double t1 = now_ns();
                check(tp_type_commit(&t));
                double t2 = now_ns();
                if (i == 0) {
                    int64_t start, counts[TP_MAX_DIMS], strides[TP_MAX_DIMS];
                    check(tp_type_get_strided_block(t, &ndims, &start, counts, strides));
                }
                tp_type_free(&t);
                t_create[i] = t1 - t0;
                t_commit[i] = t2 - t1;
            }
            printf("%s{\"type\": \"%s\", \"shape\": %d, \"canonical_dims\": %d, \"iterations\": %d, "
                   "\"create_trimean_ns\": %.1f, \"commit_trimean_ns\": %.1f}",
                   first ? "" : ", ", cases[c].name, cases[c].per_shape ? s : -1, ndims, iters,
                   trimean(t_create, iters), trimean(t_commit, iters));
            first = 0;
        }
    }
    if (argc > 2) {
        check(tp_model_load(argv[2]));
        tp_type t = b_cfg_halo_face(&shapes[0]);
        check(tp_type_commit(&t));
        const int n = 1000000;
        int method = 0, sum = 0;
        double times[3];
        check(tp_model_select(t, 1, 5e-6, 20e-6, &method, times)); /* first call interpolates, the rest hit the memo */
        double t0 = now_ns();
        for (int i = 0; i < n; ++i) {
            check(tp_model_select(t, 1, 5e-6, 20e-6, &method, times));
            sum += method;
        }
        double per = (now_ns() - t0) / n;
        printf(", {\"type\": \"tp_model_select (memoised)\", \"iterations\": %d, \"ns_per_query\": %.1f, \"method\": %d}",
               n, per, sum / n);
        tp_type_free(&t);
    }
    printf("]\n");
    free(t_create);
    free(t_commit);
    return 0;
}
