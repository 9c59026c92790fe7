/*
 * tp_pack.h - C ABI of the MI355X strided-datatype pack/unpack library.
 *
 * The library implements the datatype-handling path of the TEMPI paper
 * (arXiv 2012.14363) for one AMD CDNA4 GPU:
 *
 *   constructors (Sec. 2)  ->  commit: translate to the Type IR (Sec. 3.1),
 *   canonicalize by dense folding / stream elision / stream flattening
 *   (Sec. 3.2, Alg. 1-4), convert to one StridedBlock (Sec. 3.3, Alg. 5) and
 *   plan the kernel (Sec. 3.3)  ->  MPI_Pack / MPI_Unpack on GPU buffers
 *   (Sec. 6.2), optionally with the contiguous side in pinned host memory
 *   (the pack half of the "one-shot" method, Sec. 4).
 *
 * Conventions
 *   - Every function returns TP_SUCCESS (0) or a positive TP_ERR_* code.  On
 *     any error the out-parameters (*newtype, *position, *size, ...) are left
 *     unchanged and no data is written.  Nothing throws, nothing aborts.
 *   - All displacements, sizes and extents are bytes in int64_t.
 *   - Handles are small integers owned by the library until tp_type_free.  A
 *     derived type keeps its own reference to its oldtype, so freeing the
 *     oldtype right after construction is legal (as in MPI).
 *   - The caller owns every data buffer.  Pack and unpack allocate no device
 *     memory and the library keeps no per-type metadata on the device:
 *     everything a kernel needs travels in its kernel arguments (Sec. 3.3,
 *     last paragraph).  Only the resource cache, the staged host delivery
 *     without a caller's staging buffer and tp_model_measure allocate.
 *   - Thread safety: the handle table is guarded by a mutex; pack/unpack calls
 *     may run concurrently on distinct streams.
 *   - There is no CPU fallback: pack/unpack need a working HIP device and
 *     return TP_ERR_OTHER without one.
 */
#ifndef TP_PACK_H
#define TP_PACK_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t tp_type; /* opaque datatype handle; negative values are never valid */

#define TP_TYPE_NULL ((tp_type)-1)

/* Predefined (named) types, Sec. 2 first bullet.  Always valid and committed. */
#define TP_BYTE   ((tp_type)0)
#define TP_CHAR   ((tp_type)1)
#define TP_INT8   ((tp_type)2)
#define TP_UINT8  ((tp_type)3)
#define TP_INT16  ((tp_type)4)
#define TP_UINT16 ((tp_type)5)
#define TP_INT32  ((tp_type)6)
#define TP_UINT32 ((tp_type)7)
#define TP_INT64  ((tp_type)8)
#define TP_UINT64 ((tp_type)9)
#define TP_FLOAT  ((tp_type)10)
#define TP_DOUBLE ((tp_type)11)
#define TP_NUM_PREDEFINED 12

#define TP_ORDER_C 0
#define TP_ORDER_FORTRAN 1

#define TP_MAX_DIMS 16 /* most dimensions a StridedBlock (or a subarray) may have */

enum {
    TP_SUCCESS = 0,
    TP_ERR_TYPE = 1,     /* invalid or freed handle; or type not committed at pack/unpack time       */
    TP_ERR_COUNT = 2,    /* negative count / blocklength / incount / outcount                         */
    TP_ERR_ARG = 3,      /* null out-pointer, ndims out of [1, TP_MAX_DIMS], bad subarray box, bad order,
                            negative position or buffer size, unknown override key                    */
    TP_ERR_TRUNCATE = 4, /* *position + count*size exceeds the contiguous buffer's size               */
    TP_ERR_BUFFER = 5,   /* null data pointer with bytes to move, or memory the GPU cannot address
                            (pageable host memory, or a request that ends outside its buffer)         */
    TP_ERR_OTHER = 6,    /* HIP runtime failure (no device, launch error); see tp_error_string        */
    TP_ERR_RANGE = 7     /* a size, extent or canonical form overflows int64 or exceeds TP_MAX_DIMS   */
};

/* ---- constructors (Sec. 2: contiguous, vector/hvector, subarray) -------------------------------
 * Each stores a new handle in *newtype.  `old` may be any valid handle, committed or not.
 * Counts and blocklengths must be >= 0 (0 gives an empty type); strides may be negative.
 *
 * tp_type_contiguous:      `count` copies of old, each extent(old) bytes after the previous one.
 * tp_type_vector:          `count` blocks of `blocklength` copies of old; block starts are
 *                          `stride` * extent(old) bytes apart.
 * tp_type_create_hvector:  the same with the block stride given in bytes.
 * tp_type_create_subarray: the `subsizes` box at `starts` of an ndims-dimensional array of `sizes`
 *                          elements of old.  TP_ORDER_C: the last dimension is contiguous;
 *                          TP_ORDER_FORTRAN: the first.  The new type's lower bound is 0 and its
 *                          extent that of the whole array.  Requires 0 <= subsizes[i] <= sizes[i],
 *                          sizes[i] >= 1, 0 <= starts[i] <= sizes[i] - subsizes[i].
 * Extent of every type is ub - lb with no alignment padding.
 */
int tp_type_contiguous(int count, tp_type old, tp_type *newtype);
int tp_type_vector(int count, int blocklength, int stride, tp_type old, tp_type *newtype);
int tp_type_create_hvector(int count, int blocklength, int64_t stride_bytes, tp_type old, tp_type *newtype);
int tp_type_create_subarray(int ndims, const int sizes[], const int subsizes[], const int starts[], int order,
                            tp_type old, tp_type *newtype);

/* tp_type_commit: Sec. 3 - translate, canonicalize, convert to a StridedBlock and cache it in
 * the handle (word width, tile and grid follow at call time, when the addresses and the object
 * count are known).  Idempotent; host only; *t is not modified.
 * tp_type_free: drops the caller's reference and sets *t = TP_TYPE_NULL.  Predefined types
 * cannot be freed (TP_ERR_TYPE).  No passage of the paper: handle bookkeeping with the meaning of
 * MPI_Type_free (a type built from *t keeps working). */
int tp_type_commit(tp_type *t);
int tp_type_free(tp_type *t);

/* tp_type_size: data bytes of one object (Sec. 2: the bytes the type map selects, the sum of its
 *     block lengths).  tp_type_get_extent: lower bound and extent = ub - lb of the type map, the
 *     distance between consecutive objects of a count (Sec. 2; the library keeps size, lb and ub per
 *     node from construction, Sec. 3.1).  A subarray has lb 0 and the extent of its full array;
 *     no alignment padding is added.
 * tp_pack_size: bytes that `incount` objects occupy in the packed stream = incount * size (Sec. 6.2:
 *     the packed buffer holds the selected bytes back to back, without a header).  TP_ERR_COUNT for a
 *     negative count, TP_ERR_RANGE if the product overflows int64.
 * All three work on any valid handle, committed or not; host only. */
int tp_type_size(tp_type t, int64_t *size);
int tp_type_get_extent(tp_type t, int64_t *lb, int64_t *extent);
int tp_pack_size(int incount, tp_type t, int64_t *size);

/* ---- pack / unpack (MPI_Pack / MPI_Unpack semantics, Sec. 6.2) ---------------------------------
 * tp_pack:   object i (0 <= i < incount) has its origin at inbuf + i*extent; its bytes, in
 *            type-map order, go to outbuf + *position onward.  Requires
 *            0 <= *position and *position + incount*size <= outsize, else TP_ERR_TRUNCATE.
 *            On success *position += incount*size.
 * tp_unpack: the mirror: reads inbuf + *position onward (insize = bytes in inbuf), writes
 *            outcount objects at outbuf + i*extent; bytes of outbuf outside the type map are not
 *            touched.  Unpacking a type whose map overlaps itself is erroneous (as in MPI):
 *            which duplicate wins is unspecified.
 *
 * Memory: the typed (non-contiguous) buffer - inbuf of pack, outbuf of unpack - must be DEVICE
 * memory.  The contiguous buffer may be device memory or pinned, GPU-mapped host memory
 * (hipHostMalloc): the latter is the zero-copy path of Sec. 4.  Pageable host memory gives
 * TP_ERR_BUFFER.  So does a request that runs past its buffers: on each side the first, the
 * lowest and the highest byte the call would touch are checked to be memory of the right kind
 * (not every byte in between), so that a datatype too large for its buffer is an error here
 * rather than a memory fault on the device.  No alignment is required of any buffer, position,
 * stride or run length; speed does not depend on it beyond a few percent.  `hip_stream` is a
 * hipStream_t (NULL = the default stream).
 *
 * tp_pack / tp_unpack return after the data is complete (they synchronize the stream, as the
 * paper's timed region does, Sec. 6.3).  The *_async forms only enqueue on the stream; the
 * caller synchronizes.  A call may enqueue several kernels (a very large request is split; an
 * unpack of half a million or more tiny rows alternates read-only passes over its packed bytes with
 * the passes that store them), all on `hip_stream` and in order; none allocates or records a
 * memset, so a stream capture of the *_async forms replays from a HIP graph.
 *
 * Errors: every check (handle, count, fit, buffers, planning) comes before the first kernel is
 * enqueued, and a call that fails one of them writes nothing and leaves *position unchanged.  The
 * one error that can come later is TP_ERR_OTHER from the runtime refusing a launch or the final
 * synchronize: *position is then unchanged as well, but launches of the same call that were
 * enqueued before it may already have run, so the destination holds part of the data.
 */
int tp_pack(const void *inbuf, int incount, tp_type t, void *outbuf, int64_t outsize, int64_t *position,
            void *hip_stream);
int tp_unpack(const void *inbuf, int64_t insize, int64_t *position, void *outbuf, int outcount, tp_type t,
              void *hip_stream);
int tp_pack_async(const void *inbuf, int incount, tp_type t, void *outbuf, int64_t outsize, int64_t *position,
                  void *hip_stream);
int tp_unpack_async(const void *inbuf, int64_t insize, int64_t *position, void *outbuf, int outcount, tp_type t,
                    void *hip_stream);

/* ---- batched pack / unpack -------------------------------------------------------------------
 * n requests that share one contiguous buffer and one running position, enqueued as few kernel
 * launches as possible (one launch carries up to 40 requests of *different* datatypes; the paper,
 * Sec. 7, fuses only copies of one datatype).  The result is exactly that of n consecutive
 * tp_pack (tp_unpack) calls in order i = 0..n-1: request i moves incounts[i] objects of types[i]
 * whose typed buffer is inbufs[i] (outbufs[i]).  All requests are validated first: on any error
 * nothing is enqueued and *position is unchanged.  Same memory rules as tp_pack/tp_unpack; for
 * unpack the requests' type maps must not overlap each other.  The plain forms synchronize the
 * stream; the *_async forms only enqueue.
 */
int tp_pack_batch(int n, const void *const inbufs[], const int incounts[], const tp_type types[], void *outbuf,
                  int64_t outsize, int64_t *position, void *hip_stream);
int tp_unpack_batch(int n, const void *inbuf, int64_t insize, int64_t *position, void *const outbufs[],
                    const int outcounts[], const tp_type types[], void *hip_stream);
int tp_pack_batch_async(int n, const void *const inbufs[], const int incounts[], const tp_type types[], void *outbuf,
                        int64_t outsize, int64_t *position, void *hip_stream);
int tp_unpack_batch_async(int n, const void *inbuf, int64_t insize, int64_t *position, void *const outbufs[],
                          const int outcounts[], const tp_type types[], void *hip_stream);

/* ---- measured performance model and host delivery (Sec. 4, Eq. 1-3; Sec. 6.3) -------------------
 * When packed data has to reach host memory (to be handed to a transport that cannot read device
 * memory), it can be packed straight into pinned host memory ("one-shot", zero-copy) or packed into
 * device memory and copied ("staged"); Sec. 4 also has the "device" method, where the packed
 * device buffer itself is handed to a GPU-aware transport.  Which is fastest depends on object size
 * and contiguous block length, so the paper measures the system once and interpolates at run time.
 *
 * tp_model_measure: times six primitives on the current device - pack/unpack with the contiguous
 *     side in device memory and in pinned host memory, and plain D2H / H2D copies - each as
 *     launch + execute + synchronize (the paper's timed region), on a sparse grid of object sizes
 *     (64 B .. 4 MiB) x contiguous block lengths (1 B .. 4 KiB) of 2D objects with 512-byte pitch,
 *     and installs the table as the process-wide model.  It is the "system measurement" step, not
 *     part of the pack path: it allocates and frees its own device and pinned buffers (~2 GiB).
 * tp_model_save / tp_model_load: the table as a small text file.
 * tp_model_query: interpolated times (seconds) for `count` objects of committed type t: bilinear in
 *     (log2 bytes, log2 block) where bytes = count*size and block = the canonical contiguous run
 *     (the whole message for a dense type); block clamped to the measured range, bytes clamped below
 *     it and scaled proportionally above it.  Results are memoised.  TP_ERR_ARG if no model is loaded.
 * tp_model_select: Eq. 1-3.  t_cpu_cpu and t_gpu_gpu are the transport terms, which need a second
 *     rank to measure and are therefore inputs (seconds; 0 if unknown).  *method receives the
 *     fastest of TP_METHOD_DEVICE / ONESHOT / STAGED; times (may be NULL) the three totals.
 * tp_pack_host: tp_pack whose outbuf is pinned host memory, by the method asked for:
 *     TP_METHOD_ONESHOT, TP_METHOD_STAGED (through `staging`, caller-owned device memory of
 *     staging_size >= incount*size bytes; with staging NULL the library leases a device buffer
 *     from its resource cache for the duration of the call, see below), or TP_METHOD_AUTO
 *     (staged if the model predicts gpu_pack + d2h < host_pack, else one-shot).  A non-NULL
 *     staging that is too small is TP_ERR_ARG for STAGED and means one-shot for AUTO.
 *     Synchronizes.  *method_used (may be NULL) reports the choice.  tp_unpack_host is the mirror
 *     (host inbuf -> device typed buffer).
 */
typedef struct tp_model_times {
    double gpu_pack, gpu_unpack, host_pack, host_unpack, d2h, h2d;
} tp_model_times;

#define TP_METHOD_AUTO (-1)
#define TP_METHOD_DEVICE 0
#define TP_METHOD_ONESHOT 1
#define TP_METHOD_STAGED 2

int tp_model_measure(void *hip_stream);
int tp_model_save(const char *path);
int tp_model_load(const char *path);
int tp_model_query(tp_type t, int count, tp_model_times *out);
int tp_model_select(tp_type t, int count, double t_cpu_cpu, double t_gpu_gpu, int *method, double times[3]);
int tp_pack_host(const void *inbuf, int incount, tp_type t, void *host_outbuf, int64_t outsize, int64_t *position,
                 void *staging, int64_t staging_size, int method, void *hip_stream, int *method_used);
int tp_unpack_host(const void *host_inbuf, int64_t insize, int64_t *position, void *outbuf, int outcount, tp_type t,
                   void *staging, int64_t staging_size, int method, void *hip_stream, int *method_used);

/* tp_pack_host_static: for callers that cannot allocate - tight serving loops, harnesses that
 * forbid hipMalloc, code that runs while another thread captures a HIP graph (it synchronizes its
 * stream, so it is not itself for use on a capturing stream).  It is tp_pack_host with TP_METHOD_STAGED
 * whose staging buffer is neither the caller's nor leased: a fixed array of
 * TP_STATIC_STAGING_BYTES that is part of the library's device image (each GPU the library runs on
 * holds its own copy until the process ends).  The call gathers the objects into that array with
 * the pack kernels, copies exactly incount*size bytes from it to host_outbuf + *position with a
 * dense copy kernel, synchronizes the stream and advances *position.  It calls no hipMalloc,
 * hipFree or other allocating routine; inbuf must be device memory and host_outbuf pinned,
 * GPU-mapped host memory (or device memory), both checked as in tp_pack.
 * Errors: as tp_pack, plus TP_ERR_RANGE if incount*size exceeds TP_STATIC_STAGING_BYTES (nothing
 * is written; use tp_pack_host with a staging buffer of your own for larger messages).
 * All calls on one GPU share that GPU's array, which keeps the last call's bytes: the call itself
 * needs nothing cleared (it reads back only what it has just written), but two calls that overlap
 * in time on one GPU - from two threads, or on two streams - race on it.  Serialize them. */
#define TP_STATIC_STAGING_BYTES (4 << 20)
int tp_pack_host_static(const void *inbuf, int incount, tp_type t, void *host_outbuf, int64_t outsize,
                        int64_t *position, void *hip_stream);

/* ---- resource cache (Sec. 5) ------------------------------------------------------------------
 * A send/receive layer built on this library needs, per message, an intermediate buffer (device
 * or pinned host), often a stream and an event.  Creating them costs the runtime microseconds to
 * milliseconds; Sec. 5 serves repeated requests from a cache instead.  Resources are leased and
 * given back; a released resource stays alive and serves the next request of its kind on the
 * same device (buffers: of the same size class - capacities are rounded up to a quarter step of
 * a power of two, 4 KiB at least).  All calls are thread-safe.
 *
 * tp_resource_acquire: kind TP_RES_DEVICE (device memory), TP_RES_PINNED (page-locked host
 *     memory mapped into the device's address space, usable as the contiguous side of any
 *     pack/unpack call), TP_RES_STREAM (a hipStream_t, non-blocking, default priority) or
 *     TP_RES_EVENT (a hipEvent_t without timing).  `bytes` >= 0 is the least capacity of a buffer
 *     and ignored otherwise.  *handle receives the buffer address / stream / event, created on the
 *     calling thread's current device.  Buffer contents are whatever the last holder left.
 *     TP_ERR_ARG for a bad kind, negative bytes or NULL handle; TP_ERR_OTHER if the runtime cannot
 *     create the resource even after idle resources were freed.
 * tp_resource_release: gives a lease back.  The caller must first have waited for all device work
 *     that uses it: the next holder may get it at once.  TP_ERR_ARG if `handle` is not a current
 *     lease of that kind (never leased, or released already).
 * tp_resource_trim: destroys every idle resource; *bytes_freed (may be NULL) = buffer bytes.
 * tp_resource_stats: counters of one kind since the process started.
 * Pointers into a leased buffer are recognised by pack/unpack without the per-call
 * memory-residency query.  Nothing is freed at process exit.
 */
#define TP_RES_DEVICE 0
#define TP_RES_PINNED 1
#define TP_RES_STREAM 2
#define TP_RES_EVENT 3

typedef struct tp_resource_counts {
    int64_t hits, misses;              /* acquires served from the cache / by the runtime */
    int64_t idle, leased;              /* resources alive now */
    int64_t idle_bytes, leased_bytes;  /* buffer capacities (0 for streams and events) */
} tp_resource_counts;

int tp_resource_acquire(int kind, int64_t bytes, void **handle);
int tp_resource_release(int kind, void *handle);
int tp_resource_trim(int64_t *bytes_freed);
int tp_resource_stats(int kind, tp_resource_counts *out);

/* ---- introspection for tests and ablations ------------------------------------------------------
 * tp_type_get_strided_block: the canonical form of a committed type (Sec. 3.3): *ndims dimensions,
 * counts[0] contiguous bytes with strides[0] == 1, dimension d+1 repeats dimension d counts[d+1]
 * times strides[d+1] bytes apart; *start is the displacement of the first byte from the origin.
 * Dimensions are in nesting order (the packed stream is row-major over counts, last dimension
 * slowest), which keeps the MPI type-map order.  An empty type reports ndims 1, counts[0] 0.
 * counts/strides must have room for TP_MAX_DIMS entries.
 *
 * tp_set_override(key, value): force planner choices.  Keys:
 *   "word"          "0" (automatic) or 1, 2, 4, 8, 16: upper limit on the access width in bytes
 *   "check_buffers" "1" (default) or "0": skip the per-call memory-residency queries (then the
 *                   buffers are taken to be GPU-addressable and large enough: the caller's duty)
 *   "nt"            "-1" (automatic), 0..3, 6 or 7: streaming hints, bit 0 = non-temporal loads,
 *                   bit 1 = non-temporal stores, bit 2 (with bit 1) = the stores also written through L2 at once
 *   "ur"            "-1" (automatic), 1 or 4: rows per thread where a run fits one workgroup
 *   "xpose"         "1" (default) or "0": allow the transposing kernel (tiles through LDS for
 *                   blocks whose short elements are adjacent along an outer dimension)
 *   "narrow_partial_rows" "1" (default) or "0": unpack rows that are not whole aligned 128-byte
 *                   memory lines in narrow words (measured faster) rather than the widest
 *   "unpack_rule"   "1" (default) or "0": 0 plans such rows as before write-through stores
 *                   (4- or 8-byte words, four rows per thread), for comparisons
 *   "stage"         "-1" (automatic: from 2^19 rows), "0" (never) or "1" (wherever it applies): staged
 *                   unpack of rows of one word at 512-, 256- or 128-byte pitch (a read-only pass per chunk
 *                   of packed bytes, then the stores); "stage_bytes" 4096 .. 2^30: packed bytes per chunk
 *                   (default 16 MiB); "stage_grid" "0" (automatic) or the workgroups of such a launch (up to 2^20)
 *   "grid"          "0" (default: one workgroup per tile) or 1 .. 2^20: workgroups of every other row-by-row
 *                   launch, each then taking every grid-th tile (for measurements)
 *   "max_rows_per_launch", "max_words_per_run"  1 .. 2^30: split limits (tests lower them to
 *                   exercise the multi-launch path on small inputs)
 * tp_last_plan: describes the kernel launches of the calling thread's most recent
 * pack/unpack as text (variant, word width, grid), for tests.
 */
int tp_type_get_strided_block(tp_type t, int *ndims, int64_t *start, int64_t counts[], int64_t strides[]);
int tp_set_override(const char *key, const char *value);
const char *tp_last_plan(void);
/* tp_error_string: text for a TP_* code (for TP_ERR_OTHER the runtime's own message of the calling
 * thread's last failure).  No passage of the paper: error reporting.  The string is owned by the
 * library and valid until the thread's next failing call. */
const char *tp_error_string(int code);

#ifdef __cplusplus
}
#endif
#endif /* TP_PACK_H */
