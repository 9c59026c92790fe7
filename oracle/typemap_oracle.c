/*
 * CPU oracle, C twin of oracle/typemap.py.  TEST INFRASTRUCTURE ONLY: used by
 * the tests, the smoke check and the benchmark's cpu_baseline leg, never by
 * the product path, and it shares nothing with the HIP library.
 *
 * It interprets an MPI derived datatype as its type map, the ordered list of
 * (byte displacement, length) blocks, exactly as the constructors are defined
 * in the paper's Sec. 2 (after MPI-3.1 Sec. 4.1), and implements MPI_Pack /
 * MPI_Unpack (paper Sec. 6.2) as one memcpy per block in type-map order.  No
 * canonical form, no merging of blocks, no reordering.
 *
 * A datatype arrives as a prefix-order array of int64:
 *   NAMED      : 0, size_bytes
 *   CONTIGUOUS : 1, count, <old>
 *   VECTOR     : 2, count, blocklength, stride_elems, <old>
 *   HVECTOR    : 3, count, blocklength, stride_bytes, <old>
 *   SUBARRAY   : 4, ndims, order(0=C,1=Fortran), sizes[ndims], subsizes[ndims], starts[ndims], <old>
 *
 * Readings where the paper is silent are those listed in typemap.py's header.
 *
 * The optional threaded pack/unpack splits the outermost loop (objects, or the
 * root constructor's first loop) over plain pthreads; it is the same walk on
 * disjoint index ranges and exists only so the reported CPU baseline can use
 * the host's cores.
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define TMO_MAX_DIMS 16

enum { K_NAMED = 0, K_CONTIG = 1, K_VECTOR = 2, K_HVECTOR = 3, K_SUBARRAY = 4 };

typedef struct Node {
    int kind;
    int64_t count, blocklength, stride;          /* contiguous / vector / hvector        */
    int ndims, order;                            /* subarray                             */
    int64_t sizes[TMO_MAX_DIMS], subs[TMO_MAX_DIMS], starts[TMO_MAX_DIMS];
    int64_t named_size;
    struct Node *old;
    int64_t lb, ub, size;                        /* filled at parse time                 */
} Node;

static void node_free(Node *t) {
    if (!t) return;
    node_free(t->old);
    free(t);
}

static int64_t imin(int64_t a, int64_t b) { return a < b ? a : b; }
static int64_t imax(int64_t a, int64_t b) { return a > b ? a : b; }

/* lb/ub/size of a node from those of its child: the child occupies
 * [pos + lb_old, pos + ub_old) at every position the constructor places it. */
static void node_measure(Node *t) {
    if (t->kind == K_NAMED) {
        t->lb = 0; t->ub = t->named_size; t->size = t->named_size;
        return;
    }
    const Node *o = t->old;
    int64_t ex = o->ub - o->lb;
    if (t->kind == K_SUBARRAY) {
        int64_t total = 1, picked = 1;
        for (int e = 0; e < t->ndims; ++e) { total *= t->sizes[e]; picked *= t->subs[e]; }
        t->lb = 0; t->ub = ex * total; t->size = picked * o->size;
        return;
    }
    int64_t c = t->count, l = (t->kind == K_CONTIG) ? 1 : t->blocklength;
    t->size = c * l * o->size;
    /* no copy placed (a zero count): lb = ub = 0 */
    int64_t lb = 0, ub = 0;
    int first = 1;
    for (int64_t i = 0; i < c; ++i) {
        for (int64_t j = 0; j < l; ++j) {
            int64_t pos;
            if (t->kind == K_CONTIG) pos = i * ex;
            else if (t->kind == K_VECTOR) pos = (i * t->stride + j) * ex;
            else pos = i * t->stride + j * ex;
            if (first) { lb = pos + o->lb; ub = pos + o->ub; first = 0; }
            else { lb = imin(lb, pos + o->lb); ub = imax(ub, pos + o->ub); }
        }
    }
    t->lb = lb; t->ub = ub;
}

static Node *node_parse(const int64_t *enc, int64_t n, int64_t *pos) {
    if (*pos >= n) return NULL;
    Node *t = (Node *)calloc(1, sizeof(Node));
    if (!t) return NULL;
    t->kind = (int)enc[(*pos)++];
    int need = 0;
    switch (t->kind) {
    case K_NAMED: need = 1; break;
    case K_CONTIG: need = 1; break;
    case K_VECTOR: case K_HVECTOR: need = 3; break;
    case K_SUBARRAY: need = 2; break;
    default: free(t); return NULL;
    }
    if (*pos + need > n) { free(t); return NULL; }
    if (t->kind == K_NAMED) {
        t->named_size = enc[(*pos)++];
        node_measure(t);
        return t;
    }
    if (t->kind == K_CONTIG) {
        t->count = enc[(*pos)++];
    } else if (t->kind == K_VECTOR || t->kind == K_HVECTOR) {
        t->count = enc[(*pos)++];
        t->blocklength = enc[(*pos)++];
        t->stride = enc[(*pos)++];
    } else {
        t->ndims = (int)enc[(*pos)++];
        t->order = (int)enc[(*pos)++];
        if (t->ndims < 1 || t->ndims > TMO_MAX_DIMS || *pos + 3 * (int64_t)t->ndims > n) { free(t); return NULL; }
        for (int e = 0; e < t->ndims; ++e) t->sizes[e] = enc[(*pos)++];
        for (int e = 0; e < t->ndims; ++e) t->subs[e] = enc[(*pos)++];
        for (int e = 0; e < t->ndims; ++e) t->starts[e] = enc[(*pos)++];
    }
    t->old = node_parse(enc, n, pos);
    if (!t->old) { free(t); return NULL; }
    node_measure(t);
    return t;
}

/* ------------------------------------------------------------------ walking */
typedef struct Sink {
    void (*block)(struct Sink *, int64_t disp, int64_t len);
    /* pack / unpack */
    const uint8_t *src; uint8_t *dst;
    int64_t typed_len;       /* bytes in the typed buffer, for bounds checks   */
    int64_t p;               /* running packed offset                          */
    int error;
    /* enumeration */
    int64_t *disp_out, *len_out, cap, nblocks;
} Sink;

static void walk(const Node *t, int64_t d, Sink *s);

/* Subarray: nested loops over the selected index ranges.  C order: dimension 0
 * is the outermost loop and the last dimension is contiguous; Fortran order:
 * the reverse. */
static void walk_subarray(const Node *t, int64_t d, int level, int64_t lin, Sink *s) {
    if (level == t->ndims) {
        walk(t->old, d + lin * (t->old->ub - t->old->lb), s);
        return;
    }
    int e = (t->order == 0) ? level : t->ndims - 1 - level;
    int64_t pitch = 1;
    if (t->order == 0) { for (int f = e + 1; f < t->ndims; ++f) pitch *= t->sizes[f]; }
    else               { for (int f = 0; f < e; ++f) pitch *= t->sizes[f]; }
    for (int64_t k = 0; k < t->subs[e]; ++k)
        walk_subarray(t, d, level + 1, lin + (t->starts[e] + k) * pitch, s);
}

static void walk(const Node *t, int64_t d, Sink *s) {
    switch (t->kind) {
    case K_NAMED:
        s->block(s, d, t->named_size);
        break;
    case K_CONTIG: {
        int64_t ex = t->old->ub - t->old->lb;
        for (int64_t i = 0; i < t->count; ++i) walk(t->old, d + i * ex, s);
        break;
    }
    case K_VECTOR: {
        int64_t ex = t->old->ub - t->old->lb;
        for (int64_t i = 0; i < t->count; ++i)
            for (int64_t j = 0; j < t->blocklength; ++j)
                walk(t->old, d + (i * t->stride + j) * ex, s);
        break;
    }
    case K_HVECTOR: {
        int64_t ex = t->old->ub - t->old->lb;
        for (int64_t i = 0; i < t->count; ++i)
            for (int64_t j = 0; j < t->blocklength; ++j)
                walk(t->old, d + i * t->stride + j * ex, s);
        break;
    }
    case K_SUBARRAY:
        walk_subarray(t, d, 0, 0, s);
        break;
    }
}

/* The root constructor's first loop, restricted to iterations [lo, hi): used
 * only to hand disjoint parts of one object to different threads. */
static int64_t outer_trip_count(const Node *t) {
    switch (t->kind) {
    case K_CONTIG: case K_VECTOR: case K_HVECTOR: return t->count;
    case K_SUBARRAY: return t->subs[(t->order == 0) ? 0 : t->ndims - 1];
    default: return 1;
    }
}

static void walk_outer_range(const Node *t, int64_t d, int64_t lo, int64_t hi, Sink *s) {
    if (t->kind == K_NAMED) { if (lo == 0 && hi >= 1) walk(t, d, s); return; }
    int64_t ex = t->old->ub - t->old->lb;
    for (int64_t i = lo; i < hi; ++i) {
        if (t->kind == K_CONTIG) walk(t->old, d + i * ex, s);
        else if (t->kind == K_VECTOR)
            for (int64_t j = 0; j < t->blocklength; ++j) walk(t->old, d + (i * t->stride + j) * ex, s);
        else if (t->kind == K_HVECTOR)
            for (int64_t j = 0; j < t->blocklength; ++j) walk(t->old, d + i * t->stride + j * ex, s);
        else {
            int e = (t->order == 0) ? 0 : t->ndims - 1;
            int64_t pitch = 1;
            if (t->order == 0) { for (int f = e + 1; f < t->ndims; ++f) pitch *= t->sizes[f]; }
            else               { for (int f = 0; f < e; ++f) pitch *= t->sizes[f]; }
            walk_subarray(t, d, 1, (t->starts[e] + i) * pitch, s);
        }
    }
}

static void sink_pack(Sink *s, int64_t disp, int64_t len) {
    if (disp < 0 || disp + len > s->typed_len) { s->error = 1; return; }
    memcpy(s->dst + s->p, s->src + disp, (size_t)len);
    s->p += len;
}

static void sink_unpack(Sink *s, int64_t disp, int64_t len) {
    if (disp < 0 || disp + len > s->typed_len) { s->error = 1; return; }
    memcpy(s->dst + disp, s->src + s->p, (size_t)len);
    s->p += len;
}

static void sink_list(Sink *s, int64_t disp, int64_t len) {
    if (s->nblocks < s->cap) { s->disp_out[s->nblocks] = disp; s->len_out[s->nblocks] = len; }
    s->nblocks++;
}

/* ------------------------------------------------------------------ C entry points */
int tmo_measure(const int64_t *enc, int64_t n, int64_t *size, int64_t *lb, int64_t *ub) {
    int64_t pos = 0;
    Node *t = node_parse(enc, n, &pos);
    if (!t || pos != n) { node_free(t); return -1; }
    *size = t->size; *lb = t->lb; *ub = t->ub;
    node_free(t);
    return 0;
}

/* Writes up to cap blocks of `incount` objects; returns the total number of blocks (or -1). */
int64_t tmo_blocks(const int64_t *enc, int64_t n, int64_t incount, int64_t *disp, int64_t *len, int64_t cap) {
    int64_t pos = 0;
    Node *t = node_parse(enc, n, &pos);
    if (!t || pos != n) { node_free(t); return -1; }
    Sink s; memset(&s, 0, sizeof s);
    s.block = sink_list; s.disp_out = disp; s.len_out = len; s.cap = cap;
    for (int64_t obj = 0; obj < incount; ++obj) walk(t, obj * (t->ub - t->lb), &s);
    node_free(t);
    return s.nblocks;
}

typedef struct Job {
    const Node *t; Sink sink;
    int64_t origin, unit_lo, unit_hi, trips;   /* units = obj * trips + outer iteration */
} Job;

static void *job_run(void *arg) {
    Job *j = (Job *)arg;
    int64_t ex = j->t->ub - j->t->lb;
    int64_t u = j->unit_lo;
    while (u < j->unit_hi) {
        int64_t obj = u / j->trips, lo = u % j->trips;
        int64_t hi = imin(j->trips, lo + (j->unit_hi - u));
        walk_outer_range(j->t, j->origin + obj * ex, lo, hi, &j->sink);
        u += hi - lo;
    }
    return NULL;
}

/* direction 0: pack  (typed -> packed);  1: unpack (packed -> typed).
 * `typed` points at the start of the typed buffer of typed_len bytes; the
 * objects' origin is typed + origin.  Returns the new position, or -1 on a
 * parse error, -2 if the packed buffer is too short, -3 if a block would
 * leave the typed buffer (buffers may then be partly written). */
int64_t tmo_copy(int direction, const int64_t *enc, int64_t n, uint8_t *typed, int64_t typed_len, int64_t origin,
                 int64_t count, uint8_t *packed, int64_t packed_len, int64_t position, int nthreads) {
    int64_t pos = 0;
    Node *t = node_parse(enc, n, &pos);
    if (!t || pos != n) { node_free(t); return -1; }
    if (count < 0 || position < 0 || position + count * t->size > packed_len) { node_free(t); return -2; }
    int64_t trips = outer_trip_count(t);
    int64_t units = count * trips;
    int64_t unit_bytes = trips ? t->size / trips : 0;
    if (nthreads < 1) nthreads = 1;
    if ((int64_t)nthreads > units) nthreads = units > 0 ? (int)units : 1;
    Job *jobs = (Job *)calloc((size_t)nthreads, sizeof(Job));
    pthread_t *tids = (pthread_t *)calloc((size_t)nthreads, sizeof(pthread_t));
    int err = 0;
    for (int k = 0; k < nthreads; ++k) {
        Job *j = &jobs[k];
        j->t = t; j->origin = origin; j->trips = trips ? trips : 1;
        j->unit_lo = units * k / nthreads; j->unit_hi = units * (k + 1) / nthreads;
        j->sink.block = direction == 0 ? sink_pack : sink_unpack;
        j->sink.src = direction == 0 ? typed : packed;
        j->sink.dst = direction == 0 ? packed : typed;
        j->sink.typed_len = typed_len;
        j->sink.p = position + j->unit_lo * unit_bytes;
    }
    if (nthreads == 1) job_run(&jobs[0]);
    else {
        for (int k = 0; k < nthreads; ++k) pthread_create(&tids[k], NULL, job_run, &jobs[k]);
        for (int k = 0; k < nthreads; ++k) pthread_join(tids[k], NULL);
    }
    for (int k = 0; k < nthreads; ++k) err |= jobs[k].sink.error;
    int64_t result = err ? -3 : position + count * t->size;
    free(jobs); free(tids);
    node_free(t);
    return result;
}
