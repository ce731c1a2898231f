/*
 * bms.h -- C ABI of the MI355X-native matrix-based bulk minibatch sampler.
 *
 * The library samples k minibatches in one call ("bulk sampling", Sec. 4.1.4 / 4.2.4
 * and Eq. 1 of arxiv 2311.02909): the per-minibatch selection matrices Q are stacked,
 * P = Q A is formed against the CSR adjacency A resident in device memory, each row of
 * P is sampled by inverse-transform sampling (SAMPLE), and the sampled adjacency of
 * every layer is produced by row/column extraction (EXTRACT) -- the loop of Alg. 1.
 * Inputs follow the problem statement at the head of Sec. 4: A in {0,1}^{n x n},
 * Q^L given as the list of minibatch vertices, b, s; the output is the list of sampled
 * adjacency matrices A^0..A^{L-1}, stacked over the k minibatches.
 *
 * Conventions
 *   - Every function returns BMS_OK (0) or a negative BMS_E* code, never throws and
 *     never aborts.  On error *out is left untouched; bms_last_error() gives detail.
 *     A result passed in opts->recycle is empty after a failed call (k = L = 0, every
 *     accessor returns BMS_EINVAL); it stays valid for bms_free and for recycling again.
 *   - Hop h = 0..L-1 counts outward from the seed vertices: hop 0 is the paper's layer
 *     L (the batch vertices), params[0] applies there.
 *   - Pointers marked "device" are HIP device pointers on the current device; "host"
 *     are ordinary host pointers.  `batches` may be either (detected).
 *   - Work is enqueued on opts->stream; a call returns after the stream has drained
 *     (it reads the output sizes back), so result pointers are immediately readable
 *     by any stream that is ordered after that point.
 *   - With BMS_ASYNC a node-wise call that recycles a result of the same call shape (same csr, k, b,
 *     fanouts, variant flags) returns as soon as its kernels are enqueued: the sizes, the seed check and
 *     the device times are read when the result is first looked at -- every accessor of a result
 *     (bms_result_info / _hop / _minibatch / _minibatch_offsets / _stage, bms_aggregate_hop) and
 *     bms_result_wait first wait for the call's completion event and then report what the call would have
 *     returned: BMS_ERANGE for a bad seed, BMS_EAGAIN when the kernels gave up on the input (ids crowded
 *     into a narrow range; the result is empty, and the repeated call takes another kernel path).
 *     Ordering rules: the next sampling call on the same bms_csr must be enqueued on the same stream (it
 *     reuses the handle's scratch in stream order); other streams that read the result's buffers must be
 *     ordered after the call (bms_result_wait, or an event recorded on opts->stream after the call).
 *     Calls that do not qualify (first call of a shape, LADIES) ignore the flag and return synchronously.
 *   - A handle is not thread-safe; different handles may be used from different threads.
 *     One bms_csr must not be used by two sampling calls at the same time (it owns the
 *     scratch memory both would use).
 *   - Randomness is a stateless counter hash of (seed, hop, mb_base + minibatch index,
 *     vertex, draw index): a call is a pure function of its arguments, and one call with
 *     k minibatches equals k calls with one minibatch each and mb_base advanced.
 */
#ifndef BMS_H
#define BMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BMS_OK 0
#define BMS_EINVAL (-1)  /* null pointer, k/b/L < 1, a parameter < 1, bad hop index, unknown flag   */
#define BMS_ERANGE (-2)  /* seed vertex outside [0,n) or repeated inside one minibatch              */
#define BMS_EFORMAT (-3) /* CSR not monotone, row not strictly ascending, column outside [0,n)      */
#define BMS_ENOMEM (-4)  /* device or host allocation failed, or scratch limit too small            */
#define BMS_EHIP (-5)    /* a HIP runtime call failed                                               */
#define BMS_EAGAIN (-6)  /* deferred result of a BMS_ASYNC call: the kernel path it had enqueued gave up on  */
                         /* this input (see BMS_ASYNC); the result is empty, repeat the call                 */

/* where the arrays handed to bms_csr_load live */
#define BMS_HOST 0          /* host arrays, copied to the device                                    */
#define BMS_DEVICE_BORROW 1 /* device arrays, used in place; caller keeps them alive and unchanged  */
#define BMS_DEVICE_COPY 2   /* device arrays, copied                                                */

/* bms_opts.flags */
#define BMS_LADIES_SQUARED 1u /* LADIES column weight e_v^2 (definition in Sec. 2.2) instead of e_v   */
#define BMS_PROFILE 2u        /* record per-stage device times, see bms_result_stage                  */
#define BMS_EXTRACT_BUCKETS 4u /* node-wise EXTRACT by one workgroup per minibatch over id-range bins      */
#define BMS_EXTRACT_BITMAP 8u  /* node-wise EXTRACT by per-minibatch bitmaps in HBM (default above 2.6e8 vertices) */
#define BMS_EXTRACT_SORT 16u   /* node-wise EXTRACT by LDS sorts of id-range segments (default)              */
#define BMS_PROFILE_MAIN 64u   /* as BMS_PROFILE, but only the sampler's main kernel stage (nw_sample, ldw_accumulate)   */
#define BMS_LADIES_DENSE 32u   /* LADIES with dense per-minibatch counters in HBM instead of LDS windows     */
                               /* all give identical results; the flags only pick the kernel path          */
#define BMS_UNION_DST 128u     /* node-wise variant: the frontier's own vertices stay columns of the sampled     */
                               /* adjacency, so the next frontier = frontier + sampled vertices (what a layer    */
                               /* that also uses a vertex's own features needs); fills bms_hop_view.row_self     */
#define BMS_NODEWISE_REPLACE 256u /* node-wise variant: the s draws of a row are independent (ITS with           */
                               /* replacement: the repeat-until-distinct step of Sec. 4.1.2 left out); a row      */
                               /* keeps the distinct picks, between 1 and min(s, degree) of them                  */

#define BMS_LADIES_NO_INDEX 1024u /* LADIES by LDS windows: do not build or use the per-graph index of where adjacency */
                               /* lists cross the window boundaries (see bms_sample_ladies); same results           */
#define BMS_ASYNC 512u         /* the call may return while its kernels still run on opts->stream (see below)     */

typedef struct bms_csr bms_csr;       /* adjacency matrix on the device + reusable scratch            */
typedef struct bms_result bms_result; /* owns every device buffer its hop views point to              */

typedef struct bms_opts {   /* zero-initialised = defaults                                            */
    void *stream;           /* hipStream_t to enqueue on; NULL = the null stream                      */
    int32_t mb_base;        /* random-stream index of minibatch 0 (shards / single-minibatch replays) */
    uint32_t flags;         /* BMS_* flags above                                                      */
    bms_result *recycle;    /* result of an earlier call whose buffers may be reused; it becomes the  */
                            /* returned handle (its old contents are overwritten); NULL = allocate    */
    int64_t scratch_limit;  /* bytes of scratch the call may hold in the csr handle; 0 = 32 GiB        */
    /* Device allocator for the buffers a result exposes (e.g. one that hands out a framework's cached memory).
     * alloc returns device memory of at least `bytes` bytes, 256-byte aligned, on the current device, or NULL;
     * dealloc takes back exactly what alloc returned.  Both NULL = hipMalloc / hipFree.  A result keeps the
     * allocator it was created with (ctx must outlive it); a recycled result ignores these fields.  Scratch
     * memory in the csr handle always comes from hipMalloc. */
    void *(*alloc)(size_t bytes, void *ctx);
    void (*dealloc)(void *ptr, void *ctx);
    void *alloc_ctx;
} bms_opts;

/*
 * One hop of a bulk sample: the stacked sampled adjacency A^l of Eq. 1 in CSR form.
 * Every pointer is a device pointer owned by the result, valid until bms_free(result)
 * or until the result is recycled.
 *   rows of minibatch i   : [mb_rowoff[i], mb_rowoff[i+1])   (hop 0: i*b .. (i+1)*b, caller's order;
 *                                                             later hops: ascending vertex id)
 *   row_vertex[r]         : global vertex of stacked row r (the frontier, i.e. the nonzero of Q's row)
 *   rowptr[r]..rowptr[r+1]: entries of row r in col
 *   col[e]                : column index LOCAL to the row's minibatch, ascending inside a row
 *   col_vertex[mb_coloff[i] + c] : global vertex of local column c of minibatch i, ascending in c;
 *                           these are the rows of the next hop ("empty columns removed", Sec. 4.1.3)
 *   p_off/p_col/p_cnt     : LADIES only (else NULL, pnnz 0): the row of P = Q A of each minibatch before
 *                           normalisation, columns ascending, p_cnt = e_v (Sec. 4.2.1)
 */
typedef struct bms_hop_view {
    int64_t rows, nnz, ncols, pnnz;
    const int64_t *mb_rowoff;  /* k+1   */
    const int32_t *row_vertex; /* rows  */
    const int64_t *rowptr;     /* rows+1 */
    const int32_t *col;        /* nnz   */
    const int64_t *mb_coloff;  /* k+1   */
    const int32_t *col_vertex; /* ncols */
    const int64_t *p_off;      /* k+1   */
    const int32_t *p_col;      /* pnnz  */
    const uint32_t *p_cnt;     /* pnnz  */
    const int32_t *row_self;   /* rows: only with BMS_UNION_DST (else NULL): local column of the row's own vertex,
                                  col_vertex[mb_coloff[i] + row_self[r]] == row_vertex[r]                         */
} bms_hop_view;

/*
 * Adjacency matrix A (Sec. 4, input 1) as CSR: rowptr[n+1] int64, col[nnz] int32, each row strictly
 * ascending, entries in [0,n).  Directed patterns and self-loops are accepted.  The structure is
 * verified on the device; a violation returns BMS_EFORMAT.  `location` is one of BMS_HOST,
 * BMS_DEVICE_BORROW, BMS_DEVICE_COPY.  The handle is released with bms_free.
 */
int bms_csr_load(const int64_t *rowptr, const int32_t *col, int64_t n, int64_t nnz, int location, bms_csr **out);

/* n, nnz and the largest row length of a loaded matrix (any pointer may be NULL). */
int bms_csr_info(const bms_csr *csr, int64_t *n, int64_t *nnz, int64_t *max_degree);

/* Bytes of device memory the handle holds at this moment beyond the caller's arrays: its own copy of the matrix (if
 * it made one), the scratch of the calls made so far (kept for the next call, bounded by bms_opts.scratch_limit) and
 * the window index of bms_sample_ladies.  All of it goes back with bms_free(csr). */
int bms_csr_held_bytes(const bms_csr *csr, int64_t *bytes);

/*
 * Bulk node-wise (GraphSAGE) sampling, Sec. 4.1 with the stacking of Eq. 1.
 *   k, L    : 1 <= k <= 65535 minibatches per call, 1 <= L <= 15 hops (else BMS_EINVAL)
 *   batches : k*b seed vertices, row-major (minibatch i = batches[i*b .. (i+1)*b)), host or device;
 *             distinct inside a minibatch, each in [0,n), else BMS_ERANGE.
 *   fanouts : L host integers >= 1; fanouts[h] = s at hop h.  A row of degree <= s keeps every
 *             neighbour; otherwise exactly s distinct neighbours are chosen uniformly (ITS without
 *             replacement, Sec. 4.1.2).
 * The next hop's rows are the distinct sampled vertices of the minibatch, ascending.
 * With BMS_UNION_DST the columns of a hop are the distinct vertices among the sampled ones AND the hop's own rows
 * (ascending), so every frontier contains the one before it; which neighbours a vertex gets does not change (its
 * random stream depends on seed, hop, minibatch and vertex only).
 * With BMS_NODEWISE_REPLACE draw j of a row is floor(u_j * degree / 2^32) whatever the other draws gave, for every
 * row with degree >= 1 (also when degree <= s); the row's entries are the distinct picks.  Every fanout must then be
 * <= 2048 (BMS_EINVAL).  Both flags are node-wise only (BMS_EINVAL for LADIES) and may be combined.
 */
int bms_sample_nodewise(bms_csr *csr, const int32_t *batches, int32_t k, int32_t b, const int32_t *fanouts,
                        int32_t L, uint64_t seed, const bms_opts *opts, bms_result **out);

/*
 * Bulk layer-wise (LADIES) sampling, Sec. 4.2: per minibatch and hop, P = Q A over the whole
 * frontier (p_cnt = number of frontier vertices adjacent to the column), s_per_layer[h] draws by ITS
 * with replacement over the integer weights, duplicates removed (so ncols per minibatch <= s), then
 * the frontier's rows restricted to the sampled columns (Q_R A Q_C, Sec. 4.2.3).
 * The first call on a csr handle may build an index of the graph (for every vertex, where its sorted adjacency list
 * crosses the multiples of 2^16 in vertex id) and keep it in the handle until bms_free: n * (ceil(n / 2^16) + 1)
 * 32-bit words, built only when that is at most twice the size of the column array and a quarter of
 * opts->scratch_limit.  That call also waits for the stream once.  BMS_LADIES_NO_INDEX: neither build nor use it.
 * A call on a recycled result whose last call had the same csr, k, b, s_per_layer and weight flag waits for the
 * device only once, at its end (seed errors are reported then): its buffers are sized from what that call needed
 * plus a quarter; when that does not suffice the call repeats itself with a wait per hop (bms_result_attempts = 2).
 */
int bms_sample_ladies(bms_csr *csr, const int32_t *batches, int32_t k, int32_t b, const int32_t *s_per_layer,
                      int32_t L, uint64_t seed, const bms_opts *opts, bms_result **out);

/*
 * Completion of a BMS_ASYNC call.  bms_result_wait blocks until the call that last wrote `res` has finished and
 * returns its deferred status (BMS_OK, BMS_ERANGE, BMS_EAGAIN, BMS_EHIP); on a result that is not pending it
 * returns BMS_OK at once.  bms_result_ready returns 1 when bms_result_wait would not block, 0 when the call is
 * still running, BMS_EINVAL for a bad handle; it never blocks.
 */
int bms_result_wait(bms_result *res);
int bms_result_ready(const bms_result *res);

/* k and L of a result (either pointer may be NULL). */
int bms_result_info(const bms_result *res, int32_t *k, int32_t *L);

/* How many times the call that wrote this result enqueued its kernels: 1, or more when a kernel path gave up on
 * the input (sizes beyond what a recycled result remembered, vertex ids crowded into a narrow range) and the call
 * repeated itself on another path.  A count that stays above 1 call after call says the steady state is not reached. */
int bms_result_attempts(const bms_result *res, int32_t *attempts);

/* Fill *view for hop 0 <= hop < L. */
int bms_result_hop(const bms_result *res, int32_t hop, bms_hop_view *view);

/*
 * One minibatch of one hop, cut out of the stacked result: the k minibatches sampled in bulk are trained on one
 * after the other (Sec. 6), each with its own sampled adjacency matrices A_i.  Pointers point into the result's
 * stacked arrays (same ownership and lifetime as bms_hop_view), already moved to the minibatch's first row /
 * entry / column, so that A_i is the CSR (rowptr[r] - edge0 .. rowptr[r+1] - edge0 index `col`, r in [0, rows)).
 */
typedef struct bms_mb_view {
    int64_t rows, nnz, ncols;  /* of this minibatch                                                    */
    int64_t row0, edge0, col0; /* where it starts in the stacked rows / entries / columns of the hop   */
    const int32_t *row_vertex; /* rows   */
    const int64_t *rowptr;     /* rows+1, stacked offsets: subtract edge0                              */
    const int32_t *col;        /* nnz, local column indices (local to the minibatch as in the stack)   */
    const int32_t *col_vertex; /* ncols  */
    const int32_t *row_self;   /* rows, or NULL (see bms_hop_view)                                     */
} bms_mb_view;

/*
 * Fill *view for minibatch 0 <= i < k of hop 0 <= hop < L.  The first call on a result copies the per-minibatch
 * offsets of every hop to the host (three arrays of k+1 integers per hop; it waits for that copy); later calls on
 * the same result only do pointer arithmetic.  BMS_EINVAL for a bad handle, hop or minibatch index.
 */
int bms_result_minibatch(bms_result *res, int32_t hop, int32_t i, bms_mb_view *view);

/*
 * For callers that cannot allocate (tight serving loops, harnesses that forbid hipMalloc, code that runs while
 * another thread captures a HIP graph): the per-minibatch offsets of one hop -- the row0 / edge0 / col0 values of
 * bms_result_minibatch for every minibatch at once -- copied into caller-owned host arrays of k+1 integers each:
 *   row_off[i]  = first stacked row of minibatch i      (row_off[k]  = rows of the hop)
 *   edge_off[i] = first entry of minibatch i in `col`   (edge_off[k] = nnz of the hop)
 *   col_off[i]  = first stacked column of minibatch i   (col_off[k]  = ncols of the hop)
 * Unlike bms_result_minibatch (whose first call on a result allocates a device buffer and a host table) this call
 * allocates nothing, on the device or on the host: its one kernel writes into a fixed array of BMS_NOALLOC_MAX_K + 1
 * integers that the library holds on every GPU it runs on (128 KB, until the process ends).  k > BMS_NOALLOC_MAX_K
 * gives BMS_EINVAL.  The work is enqueued on `stream` (hipStream_t, NULL = the null stream) and the call returns
 * after the copies have completed.  All calls on one GPU share that array: calls that overlap on one GPU (two
 * threads, two streams) race and must be serialised by the caller.  The result's device must be the current device.
 */
#define BMS_NOALLOC_MAX_K 16383
int bms_result_minibatch_offsets(const bms_result *res, int32_t hop, int64_t *row_off, int64_t *edge_off,
                                 int64_t *col_off, void *stream);

/*
 * Feature fetching, the part one GPU does (Sec. 6.2): H_i = the rows of the feature matrix H that belong to
 * the vertices of the last frontier.  out[j * f + x] = H[ids[j] * f + x] for j in [0, m), x in [0, f).
 *   H    device, n x f fp32, row-major, caller-owned, read only
 *   ids  device, m vertex ids, e.g. bms_hop_view.col_vertex of the last hop (all minibatches stacked:
 *        minibatch i owns rows [mb_coloff[i], mb_coloff[i+1]) of out)
 *   out  device, m x f fp32, caller-owned, overwritten
 * The copy is enqueued on `stream` (hipStream_t, NULL = the null stream); the call returns after it has
 * completed.  Rows are copied bit for bit.  An id outside [0, n) gives BMS_ERANGE (its row is written as
 * zeros, the other rows are valid); n < 0, f < 1, m < 0, or a null pointer while m > 0, give BMS_EINVAL.
 * May be called from several threads at once (each call has its own error flag; up to 64 calls may be in
 * flight per device).
 */
int bms_fetch_features(const float *H, int64_t n, int32_t f, const int32_t *ids, int64_t m, float *out,
                       void *stream);

/*
 * Forward neighbourhood aggregation of one hop (Sec. 6.2: the SpMM between a minibatch's sampled adjacency
 * matrix A_i and the feature rows H_i of its columns), for all k minibatches of the stacked result at once.
 * For stacked row r of minibatch i:  out[r, :] = sum over the row's entries e of X[mb_coloff[i] + col[e], :],
 * divided by the number of entries when mean != 0 (every entry of A_i is 1); a row without entries gives zeros.
 *   res, hop  a completed bulk sample and the hop whose adjacency is used
 *   X         device, ncols x f fp32 row-major: one row per stacked column of the hop (for the last hop the
 *             output of bms_fetch_features on col_vertex; for earlier hops the previous aggregation's output)
 *   out       device, rows x f fp32, caller-owned, overwritten
 * fp32 arithmetic, entries added in ascending order (the result does not depend on the launch shape).
 * Enqueued on `stream`; returns without waiting.  BMS_EINVAL for a bad handle, hop, f < 1 or null pointers.
 */
int bms_aggregate_hop(const bms_result *res, int32_t hop, const float *X, int32_t f, int mean, float *out,
                      void *stream);

/*
 * Per-stage device time of the call that produced `res` (only with BMS_PROFILE; measured with HIP
 * events on the call's stream).  idx enumerates the recorded stages in launch order; returns
 * BMS_EINVAL past the end.  *name points to a static string such as "nw_sample", *hop to the hop.
 */
int bms_result_stage(const bms_result *res, int32_t idx, const char **name, int32_t *hop, float *ms);

/* Release a bms_csr or a bms_result (told apart by a tag in the handle); NULL is a no-op. */
void bms_free(void *csr_or_result);

/* Static description of an error code. */
const char *bms_strerror(int code);

/* Detail of the last error raised on the calling thread ("" if none). */
const char *bms_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* BMS_H */
