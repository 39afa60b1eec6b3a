/* pipad.h - C ABI of the frame-parallel GCN aggregation library for AMD MI355X (gfx950).
 *
 * The library implements one thing: neighbour aggregation of a GCN layer over a frame (sliding
 * window) of k graph snapshots, the way PiPAD's "dimension-aware parallel GNN" organises it
 * (Section 4.2): the topology of the snapshot group is regrouped as ONE overlap part shared by all
 * k snapshots plus one exclusive part per snapshot (Section 4.1, "Overlap-aware data transfer");
 * the overlap part is applied once to the features of all k snapshots (the "coalescent" features),
 * and every snapshot's exclusive part is applied to its own features and added back.  The result
 * is, for every snapshot t of the frame,
 *
 *      Y_t = D_t^-1/2 (A_t + I) D_t^-1/2  X_t ,      D_t = row sums of (A_t + I)
 *
 * (Eq. 1 of Section 2.1 aggregates over N(v) united with {v}; the normalisation is the symmetric
 * GCN one).  A_t is a 0/1 pattern; self-loops are implicit and never stored.
 *
 * Conventions that hold for every call
 *  - All array arguments named "device" are pointers into GPU memory of the CURRENT HIP device;
 *    arrays named "host" are ordinary host arrays that only need to live for the duration of the
 *    call.  The library never copies feature data to the host.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on
 *    that stream; the caller orders its own work against it.
 *  - Every function returns 0 (PIPAD_OK) or a negative pipad_status; nothing throws or aborts.
 *    On failure no output argument is written.
 *  - Indices are int32.  A snapshot must have fewer than 2^31 stored entries.
 */
#ifndef PIPAD_H_
#define PIPAD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PIPAD_MAX_K 32 /* most snapshots one frame may hold */

typedef enum pipad_status {
  PIPAD_OK = 0,
  PIPAD_ERR_INVALID_ARG = -1, /* null pointer, k < 1 or > PIPAD_MAX_K, n < 0, F < 1, ld < F ... */
  PIPAD_ERR_BAD_CSR = -2,     /* PIPAD_VALIDATE found a snapshot that is not canonical          */
  PIPAD_ERR_ALLOC = -3,       /* device allocation failed (callback returned NULL / hipMalloc)  */
  PIPAD_ERR_TOO_LARGE = -4,   /* a size does not fit the int32 index space                      */
  PIPAD_ERR_HIP = -5,         /* a HIP runtime call failed; see pipad_last_hip_error()          */
  PIPAD_ERR_SCRATCH = -6      /* the partial sums of this frame and F do not fit the scratch     *
                               * buffer and it cannot grow now (pipad_frame_aggregate_static; any *
                               * aggregation under stream capture); nothing was enqueued         */
} pipad_status;

/* One sparse 0/1 pattern in CSR.  Used for the input snapshots and for borrowed views of a
 * frame's parts.  Canonical form (required of inputs, guaranteed for outputs):
 * rowptr[0] == 0, rowptr non-decreasing, rowptr[n] == nnz, column indices in [0, n), strictly
 * ascending within a row, no diagonal entry. */
typedef struct pipad_csr {
  int32_t n;             /* rows == columns == number of nodes          */
  int32_t nnz;           /* stored entries == rowptr[n]                 */
  const int32_t *rowptr; /* device, int32[n + 1]                        */
  const int32_t *colidx; /* device, int32[nnz] (may be NULL when nnz=0) */
} pipad_csr_t;

/* Opaque frame: overlap CSR + k exclusive CSRs + per-snapshot D^-1/2 + launch metadata. */
typedef struct pipad_frame pipad_frame_t;

/* Optional device allocator.  Must return memory of at least `bytes` bytes, aligned to 256 bytes,
 * usable on `stream`'s device, or NULL on failure.  Memory obtained through the callback is owned
 * by the caller and must stay valid until pipad_frame_destroy(); the library never frees it.  The
 * callback and its ctx must stay callable until then too: besides the frame's own buffers it
 * serves the temporaries of the build (which the caller may take back early, see
 * pipad_frame_temporaries) and the scratch buffer of pipad_frame_aggregate. */
typedef void *(*pipad_alloc_fn)(size_t bytes, void *ctx);

#define PIPAD_VALIDATE 1u /* flag: check on the device that every input snapshot is canonical */

/* Overlap extraction (Section 4.1 "Overlap-aware data transfer", Section 4.3 data preparation
 * module): splits the k snapshots of a frame into
 *      common  = the directed edges present in every snapshot   (exact set intersection), and
 *      delta_t = edges of snapshot t that are not in common      (t = 0 .. k-1),
 * both as canonical CSR, and computes dinv_t[i] = (1 + |row i of A_t|)^-1/2.
 *
 *   n       number of nodes (same for all snapshots), n >= 0
 *   k       snapshots in the frame, 1 <= k <= PIPAD_MAX_K
 *   snaps   host array of k descriptors whose rowptr/colidx are device arrays; each must have
 *           snaps[t].n == n.  The inputs are only read and need not outlive the call.
 *   flags   0 or PIPAD_VALIDATE (costs one extra pass; returns PIPAD_ERR_BAD_CSR on violation;
 *           without it, non-canonical input gives undefined results but no out-of-range write
 *           as long as rowptr is a valid offset array into colidx)
 *   alloc   NULL: the library allocates with hipMalloc and frees in pipad_frame_destroy();
 *           otherwise every device buffer is obtained through alloc(bytes, ctx) and no
 *           hipMalloc / hipFree is issued
 *   stream  stream the kernels run on.  The call synchronises with it once (sizes of the outputs
 *           are data dependent and are read back; PIPAD_VALIDATE adds a second synchronisation).  With alloc == NULL the frame is complete on
 *           return; with a callback the last kernels may still be running on `stream`, so the
 *           inputs must stay valid, and the frame is used, in stream order.
 *   out     receives the new frame.
 */
int pipad_frame_build_overlap(int32_t n, int32_t k, const pipad_csr_t *snaps, uint32_t flags,
                              pipad_alloc_fn alloc, void *alloc_ctx, void *stream,
                              pipad_frame_t **out);

/* With a caller allocator, one of the buffers a build (or pipad_frame_transpose) obtained holds
 * only temporaries: the frame never touches it again once the work that the build enqueued on its
 * stream has completed.  This call reports that buffer (*ptr, *bytes as requested from the
 * callback; NULL / 0 with the library's own allocator, which frees its temporaries itself, or
 * when it was already taken) and the frame forgets it: the caller may release it after a
 * stream-ordered point behind the build, long before pipad_frame_destroy(). */
int pipad_frame_temporaries(pipad_frame_t *frame, void **ptr, size_t *bytes);

/* Row stride, in floats, that the feature matrices X should have when their rows are gathered
 * by pipad_frame_aggregate.  Rows of up to 128 bytes: the smallest power of two >= F, so that no
 * row straddles two 128-byte lines and nothing more is padded (F = 6 -> 8, F = 16 -> 16,
 * F = 20 -> 32; padding such rows to a whole line was measured 15-50 % slower).  Longer rows:
 * the smallest ODD number of 128-byte lines that holds F floats (F = 64 -> 96, F = 128 -> 160).
 * The call works with any ldx >= F; but with a power-of-two stride of several lines the memory
 * channel of a row is decided by a few bits of the node id, and when popular nodes share those
 * bits (ids of R-MAT-like generators do) their rows crowd onto a few channels: measured on a
 * 1M-node R-MAT frame at F = 64, ldx = 64 is 1-5 % slower than ldx = 96.  The padding is never
 * read.  Returns a negative pipad_status for F < 1. */
int64_t pipad_recommended_row_stride(int32_t F);

/* Borrowed views (valid until the frame is destroyed) of the overlap part and of the exclusive
 * part of snapshot t; see pipad_csr_t for the guarantees. */
int pipad_frame_common(const pipad_frame_t *frame, pipad_csr_t *view);
int pipad_frame_delta(const pipad_frame_t *frame, int32_t t, pipad_csr_t *view);

/* Borrowed view of D^-1/2: the value for node i of snapshot t is dinv[i * ld_node + t * ld_snap]
 * (device, float). */
int pipad_frame_dinv(const pipad_frame_t *frame, const float **dinv, int64_t *ld_node,
                     int64_t *ld_snap);

/* Frame size queries: *n, *k as given to build; each may be NULL. */
int pipad_frame_shape(const pipad_frame_t *frame, int32_t *n, int32_t *k);

/* Frame-parallel aggregation (Section 4.2 "Dimension-aware parallel GNN": parallel aggregation of
 * the overlap part with the coalescent features plus the per-snapshot aggregations of the
 * exclusive parts; Eq. 1 for what is aggregated):
 *
 *      Y[t][i, 0:F] = dinv_t[i] * ( sum_{j in common(i) U delta_t(i) U {i}} dinv_t[j] * X[t][j, 0:F] )
 *
 *   F    feature columns, F >= 1
 *   X    host array of k device pointers; X[t] is a row-major float matrix, n rows, row stride ldx
 *        elements (ldx >= F).  Passing X[t] = base + t*F with ldx = k*F hands over the physically
 *        concatenated (coalescent) operand through the same call.
 *   Y    host array of k device pointers, row stride ldy >= F; written exactly once per element
 *        (columns >= F of a wider row are not touched).  Y must not overlap X.
 *   The current HIP device must be the one the frame was built on (else PIPAD_ERR_INVALID_ARG).
 *   The frame is only read, except for its scratch buffer (hence the non-const pointer): the
 *   partial sums of rows that are summed in several parts go through it.  The first call of a
 *   frame, and any call with a larger k*F than all before, allocates it (through the frame's
 *   allocator; with the library's own allocator a buffer that is replaced is freed after a
 *   hipDeviceSynchronize).  All other calls only enqueue kernels on `stream`, without host
 *   synchronisation, so they can be recorded into a HIP graph (stream capture) once an eager call
 *   with the same or a larger k*F has sized the scratch; a call that would have to allocate while
 *   `stream` is being captured returns PIPAD_ERR_SCRATCH with nothing enqueued.
 *   Two aggregations of the SAME frame must not run concurrently (they share that scratch).
 *   Results are deterministic: same inputs, same bits.
 */
int pipad_frame_aggregate(pipad_frame_t *frame, int32_t F, const float *const *X, int64_t ldx,
                          float *const *Y, int64_t ldy, void *stream);

/* pipad_frame_aggregate for some of the frame's snapshots only: the inter-frame reuse of Section
 * 3.3 ("opportunities for data reuse") and Section 4.4 ("inter-frame reuse").  When the frame
 * slides by one snapshot, k - 1 of its snapshots were already part of the previous frame, and an
 * aggregation whose input does not depend on the weights (the first layer's) has the same result
 * for them as before: the caller keeps those Y_t and asks for the entering snapshot alone, while
 * later layers call pipad_frame_aggregate on the same frame for all k.
 *   nsel, snapshots   host array of nsel distinct snapshot numbers in [0, k), taken in this order;
 *                     nsel = 0 does nothing
 *   X, Y              host arrays of k device pointers as for pipad_frame_aggregate; only the
 *                     entries of the chosen snapshots are looked at (the others may be NULL)
 * Every chosen Y[t] gets exactly the bits pipad_frame_aggregate would give it.  Other rules
 * (device, stream, scratch, determinism) as for pipad_frame_aggregate; operands of F < 32 take
 * the per-snapshot kernel here, never the coalescent one. */
int pipad_frame_aggregate_subset(pipad_frame_t *frame, int32_t nsel, const int32_t *snapshots,
                                 int32_t F, const float *const *X, int64_t ldx, float *const *Y,
                                 int64_t ldy, void *stream);

/* pipad_frame_aggregate for callers that cannot allocate device memory: code under HIP graph
 * (stream) capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results, but the partial sums of split rows go to a fixed array of
 * PIPAD_STATIC_SCRATCH_BYTES that is part of the library's device code (every GPU the library
 * runs on holds its own copy until the process ends) instead of the frame's growable buffer, and
 * the allocator callback is never called.  The call issues no hipMalloc / hipFree and no other
 * allocating routine; the array's address on a device is looked up once, at the first
 * pipad_frame_build_overlap or pipad_frame_aggregate_static on that device.
 *   The partial sums of one snapshot take (units of rows longer than "mid_max") * (column
 *   classes) * (F rounded up to the slice width) floats.  When the array cannot hold those of all
 *   k snapshots at once the call goes through the snapshots in groups that fit, one launch after
 *   the other on `stream` (same bits); when it cannot hold one snapshot's it returns
 *   PIPAD_ERR_SCRATCH with nothing enqueued.  (The 1M-node benchmark frame at F = 64: 17 MB per
 *   snapshot, groups of 3.)
 *   All calls on one GPU share the array: calls that overlap in time on that GPU (different
 *   streams, or different frames) race on it and give wrong results; calls ordered on one stream
 *   are safe.  Nothing in the array has to be cleared between calls: every partial sum is written
 *   before it is read within the same call. */
#define PIPAD_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int pipad_frame_aggregate_static(const pipad_frame_t *frame, int32_t F, const float *const *X,
                                 int64_t ldx, float *const *Y, int64_t ldy, void *stream);

/* One GCN layer for every snapshot of the frame: the aggregation above followed by the update of
 * Eq. 1, a fully connected layer whose weights all snapshots of the frame share (Section 2.1;
 * "locality-optimized weight reuse", Section 4.2: the weights stay on chip while the rows of all
 * snapshots pass by):
 *
 *      H[t][i, 0:Fo] = ( sum_f A[t][i, f] * W[f, 0:Fo] ) + bias[0:Fo],   A[t] = the Y[t] of
 *      pipad_frame_aggregate for the same frame, F, X.
 *
 *   X, ldx, F   as for pipad_frame_aggregate
 *   W      device, row-major float [F][Fo], row stride ldw >= Fo
 *   bias   device float [Fo], or NULL for none
 *   Fo     output columns, Fo >= 1
 *   A      host array of k device pointers receiving the aggregation results (row stride lda >= F),
 *          or NULL when they are not wanted.  NULL is only possible where the update is fused
 *          into the aggregation kernel: F and Fo multiples of 4 resp. 16 with 16 <= F, Fo <= 64,
 *          16-byte aligned X (and A) with ldx (lda) a multiple of 4, and a snapshot matrix below
 *          4 GiB.  Other shapes run the aggregation into A and then a separate multiplication;
 *          without A they return PIPAD_ERR_INVALID_ARG.
 *   H      host array of k device pointers, row stride ldh >= Fo; written once per element.
 *          H, A, X, W must not overlap.
 *   Stream, device, scratch and determinism rules are those of pipad_frame_aggregate.
 */
int pipad_frame_aggregate_update(pipad_frame_t *frame, int32_t F, const float *const *X,
                                 int64_t ldx, const float *W, int64_t ldw, const float *bias,
                                 int32_t Fo, float *const *A, int64_t lda, float *const *H,
                                 int64_t ldh, void *stream);

/* The frame of the transposed patterns with the same normalisation: aggregating with `*out`
 * multiplies by the transpose of D_t^-1/2 (A_t + I) D_t^-1/2, the operator of the backward pass
 * (Eq. 1 differentiated; D_t keeps the row sums of A_t + I of the ORIGINAL snapshots).  For
 * symmetric patterns the result equals the input frame and the call is not needed.
 *
 *   frame   a frame built on the current device; not modified, may be destroyed afterwards
 *   alloc, alloc_ctx, stream   as for pipad_frame_build_overlap (one host synchronisation)
 *   out     receives the new frame: its common / exclusive parts are the transposes of `frame`'s
 *           (canonical CSR again), its D^-1/2 is a copy.
 * Errors as for pipad_frame_build_overlap; *out is untouched on failure. */
int pipad_frame_transpose(const pipad_frame_t *frame, pipad_alloc_fn alloc, void *alloc_ctx,
                          void *stream, pipad_frame_t **out);

/* Releases the frame and every buffer the library allocated itself.  NULL is allowed. */
void pipad_frame_destroy(pipad_frame_t *frame);

/* Static text for a status code. */
const char *pipad_strerror(int status);

/* Text of the last HIP runtime error seen by the calling thread ("" if none). */
const char *pipad_last_hip_error(void);

/* Tuning knobs; process-wide, not thread-safe.  A frame takes a copy of all of them when it is
 * built (pipad_frame_build_overlap; a transposed frame inherits its source's) and never looks at
 * the process-wide values again, so changing a knob affects frames built afterwards only.
 * Unknown keys, negative values and values beyond a key's range return PIPAD_ERR_INVALID_ARG.
 * Keys (row lengths count common + longest exclusive entries of a row; at most 2^30):
 *   "short_max"      rows with at most this many entries are walked whole by one small lane team,
 *                    several rows per wave (default 64)
 *   "mid_max"        rows up to this length are walked whole by one wave; longer rows ("hub rows")
 *                    are stored a second time with their entries grouped by a hash class of the
 *                    column, and the part of a row in class x is walked on XCD x only, whose L2
 *                    then caches just that class's rows of X; the 8 partial sums per row are added
 *                    up in a fixed order by a second kernel (default 512; below short_max: as
 *                    short_max)
 *   "hub_threshold"  hub rows with more entries than this are first cut into units (default 2048)
 *   "hub_segment"    entries per unit of a cut row (default 2048)
 *   "sub_classes"    column classes per XCD, 1, 2 or 4 (other values are rounded down to these):
 *                    with more than one, the hub rows are walked in that many passes per
 *                    snapshot, each pass over a smaller share of X (default 1: on MI355X the passes
 *                    read less from memory but take longer)
 *   "agg_order"      order of the workgroups of one call.  1: the slices (64 columns of one
 *                    snapshot) one after the other, so that the caches hold one snapshot's
 *                    matrix at a time; 0: the same rows of all slices side by side, so that the
 *                    slices share the entry lists they have in common (the overlap part is read
 *                    once for all snapshots); 2 (default): 0 while one slice's matrix is smaller
 *                    than 28 MiB, else 1.  Results do not depend on it.
 *   "agg_nt"         bit 0: non-temporal stores for Y (every element is written once and not read
 *                    again by the call: measured 1-2 % faster); bit 1: non-temporal loads for the
 *                    index and scale streams (no gain measured) (default 1)
 *   "slice_cols"     feature columns per slice, 1..64 (default 0 = 64)
 *   "agg_generic"    1 forces the bounds-checked kernel with 64-bit addresses (default 0: only for
 *                    matrices of 4 GB and more)
 *   "agg_coalescent" kernel for F < 32 on the concatenated operand that gathers the rows of
 *                    several snapshots with one access: 0 never, 1 automatic (default: whenever
 *                    the operand allows it and holds at least 1 MB), 2 whenever the operand
 *                    allows it
 */
int pipad_set_option(const char *key, int64_t value);
int pipad_get_option(const char *key, int64_t *value);

#ifdef __cplusplus
}
#endif
#endif /* PIPAD_H_ */
