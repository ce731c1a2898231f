// C ABI of libbms.so: handle management and the per-hop orchestration of the kernels.
#include "../../include/bms.h"
#include "bms_device.h"
#include "bms_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace bms;

// Scratch of bms_result_minibatch_offsets (the entry point that allocates nothing); see scratch_address().
static __device__ __align__(256) int64_t scratch[BMS_NOALLOC_MAX_K + 1];

namespace {

constexpr uint32_t kTagCsr = 0x31525343u;    // "CSR1"
constexpr uint32_t kTagResult = 0x31534552u; // "RES1"
constexpr int64_t kDefaultScratchLimit = 32LL << 30;
constexpr int32_t kMaxMinibatches = 65535; // some kernels take the minibatch from the second grid dimension
constexpr int64_t kNoWaitEntries = 32LL << 20; // result buffers up to this many entries may be sized by a bound
constexpr double kBitmapIdsPerEntry = 128.0; // EXTRACT ranks by bitmap when a minibatch samples at least n / this many ids
                                            // (measured: by bitmap wins at 4..15 ids of [0, n) per sampled id, by counting at 580)
constexpr int64_t kScanTmpLen = 1 << 17; // partial sums of multi-workgroup scans: arrays up to 2^29 values

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                                                  \
    do {                                                                                                               \
        hipError_t e_ = (expr);                                                                                        \
        if (e_ != hipSuccess)                                                                                          \
            return fail(e_ == hipErrorOutOfMemory ? BMS_ENOMEM : BMS_EHIP, "%s failed: %s (%s:%d)", #expr,             \
                        hipGetErrorString(e_), __FILE__, __LINE__);                                                    \
    } while (0)

#define BMS_TRY(expr)                                                                                                  \
    do {                                                                                                               \
        int rc_ = (expr);                                                                                              \
        if (rc_ != BMS_OK)                                                                                             \
            return rc_;                                                                                                \
    } while (0)

// Where a result's buffers come from (bms_opts.alloc / dealloc / alloc_ctx); both null = hipMalloc / hipFree
struct Allocator {
    void *(*alloc)(size_t, void *) = nullptr;
    void (*dealloc)(void *, void *) = nullptr;
    void *ctx = nullptr;
};

// Growable device buffer; contents are not preserved across growth.
struct DevBuf {
    void *p = nullptr;
    size_t cap = 0;
    bool grew = false; // set when the last ensure() reallocated
    const Allocator *al = nullptr; // not null: the caller's allocator (buffers a result exposes)
    DevBuf() = default;
    // a buffer that belongs to a handle enters the handle's list, which is what bms_free walks
    explicit DevBuf(std::vector<DevBuf *> *owner_list) { owner_list->push_back(this); }
    DevBuf(const DevBuf &) = delete;
    DevBuf &operator=(const DevBuf &) = delete;
    DevBuf(DevBuf &&o) noexcept : p(o.p), cap(o.cap), grew(o.grew), al(o.al) { o.p = nullptr; o.cap = 0; } // hop buffers in a vector
    void drop()
    {
        if (!p)
            return;
        if (al && al->dealloc)
            al->dealloc(p, al->ctx);
        else
            (void)hipFree(p);
        p = nullptr;
        cap = 0;
    }
    int ensure(size_t bytes)
    {
        grew = false;
        if (bytes <= cap && p)
            return BMS_OK;
        drop();
        if (bytes < 256)
            bytes = 256;
        if (al && al->alloc) {
            p = al->alloc(bytes, al->ctx);
            if (!p)
                return fail(BMS_ENOMEM, "the caller's allocator returned no memory for %zu bytes", bytes);
        } else {
            HIP_TRY(hipMalloc(&p, bytes));
        }
        cap = bytes;
        grew = true;
        return BMS_OK;
    }
    void release() { drop(); }
    template <class T>
    T *as() const
    {
        return static_cast<T *>(p);
    }
};

// Scratch of the entry point that allocates nothing (bms_result_minibatch_offsets): one array per GPU, held until
// the process ends.  Its name is only a host-side handle: the device address comes from hipGetSymbolAddress, once
// per device, and that pointer is what kernels and copies get.
constexpr int32_t kNoAllocMaxK = BMS_NOALLOC_MAX_K;
constexpr int kMaxDevices = 64;
int64_t *g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_lock;

// Device address of `scratch` on `device`, which must be the current device.
int scratch_address(int device, int64_t **out)
{
    if (device < 0 || device >= kMaxDevices)
        return fail(BMS_EINVAL, "device ordinal %d not supported", device);
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[device]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p)
            return fail(BMS_EHIP, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[device] = static_cast<int64_t *>(p);
    }
    *out = g_scratch_ptr[device];
    return BMS_OK;
}

struct StageTime {
    const char *name;
    int32_t hop;
    hipEvent_t t0, t1;
    float ms;
};

} // namespace

struct bms_csr {
    uint32_t tag = kTagCsr;
    int device = 0;
    int num_cu = 256;
    int64_t n = 0, nnz = 0, max_degree = 0;
    const int64_t *rowptr = nullptr;
    const int32_t *col = nullptr;
    std::vector<DevBuf *> bufs; // every device buffer below registers here (declared first: built first)
#define BMS_BUF(name) DevBuf name{&bufs}
    BMS_BUF(own_rowptr); BMS_BUF(own_col);
    // scratch reused across calls
    BMS_BUF(vs_words); BMS_BUF(vs_prefix); BMS_BUF(vs_chunks);
    bool vs_clean = false; // all words zero
    BMS_BUF(row_beg); BMS_BUF(row_deg); BMS_BUF(tile_off); BMS_BUF(mb_tileoff); BMS_BUF(scalars); BMS_BUF(scan_tmp);
    BMS_BUF(ld_counters); BMS_BUF(ld_gather_off); BMS_BUF(ld_row_mb); BMS_BUF(ld_chunks); BMS_BUF(ld_prefix);
    BMS_BUF(ld_ptileoff); BMS_BUF(ld_tilesum);
    BMS_BUF(dd_pairs); BMS_BUF(dd_utmp); BMS_BUF(dd_uniq); BMS_BUF(dd_edgeoff); BMS_BUF(dd_count); BMS_BUF(dd_back);
    BMS_BUF(dd_tileoff); BMS_BUF(dd_cursor); BMS_BUF(dd_seg); BMS_BUF(dd_runs); BMS_BUF(dd_segcnt); BMS_BUF(dd_done); BMS_BUF(dd_hist); // EXTRACT
    bool segcnt_clean = false; // every segment counter zero (kept so by the kernels; lost when a call is interrupted)
    BMS_BUF(un_rowptr); BMS_BUF(un_col); // BMS_UNION_DST: the hop's CSR while its rows still carry their own vertex
    BMS_BUF(row_cnt);                    // BMS_NODEWISE_REPLACE with a fanout above 32: distinct picks per row
    BMS_BUF(lw_bounds); BMS_BUF(lw_win); BMS_BUF(lw_tmpcol); BMS_BUF(lw_parts); BMS_BUF(lw_sel); BMS_BUF(lw_xtmp);
    BMS_BUF(lw_count); BMS_BUF(lw_tiles); BMS_BUF(lw_rowcnt); // LADIES by LDS windows
    BMS_BUF(lw_index);           // where every vertex's adjacency list crosses the window boundaries: n * (nwin + 1)
    bool lw_index_ready = false; // built by the first layer-wise call that finds room for it
    bool lw_index_tried = false;
#undef BMS_BUF
    bool ld_clean = false; // all dense counters zero
    int64_t *host_pinned = nullptr; // 64 int64
};

struct HopBufs {
    DevBuf mb_rowoff, row_vertex; // own storage only at hop 0; later hops alias the previous hop's columns
    DevBuf rowptr, col, mb_coloff, col_vertex, p_off, p_col, p_cnt, row_self;
    DevBuf seg_tab; // node-wise EXTRACT with segments of unequal width: cell -> segment table, then the segments' first cells
    bms_hop_view view;
    void bind(const Allocator *al) // the buffers the hop views point to come from the result's allocator
    {
        for (DevBuf *b : {&mb_rowoff, &row_vertex, &rowptr, &col, &mb_coloff, &col_vertex, &p_off, &p_col, &p_cnt, &row_self})
            if (!b->p)
                b->al = al;
    }
};

// what a BMS_ASYNC node-wise call leaves for the first look at its result
struct PendingNodewise {
    bms_csr *csr = nullptr;
    int32_t k = 0, b = 0, L = 0;
    bool union_dst = false;
    std::vector<int32_t> shape;
    std::vector<uint8_t> mode;
    std::vector<int32_t> table_built;
};

struct bms_result {
    uint32_t tag = kTagResult;
    int32_t k = 0, L = 0;
    int device = 0;
    std::vector<HopBufs> hops;
    std::vector<StageTime> stages;
    std::vector<hipEvent_t> event_pool;
    size_t events_used = 0;
    // sizes the previous node-wise call with the same shape produced; a recycled result lets the
    // next call enqueue every hop without waiting for the device (buffers sized by upper bounds)
    const bms_csr *hint_csr = nullptr;
    std::vector<int32_t> hint_shape; // k, b, fanouts...
    std::vector<int64_t> hint_nnz;   // per hop
    int32_t attempts = 1; // how often the call that wrote this result enqueued its kernels
    std::vector<int64_t> hint_gathered, hint_pnnz; // per hop, layer-wise calls: gathered neighbours D, nnz(P)
    // how each hop's EXTRACT went before: 0 = segments of equal width did, 1 = ids crowd parts of [0, n): segments of
    // unequal width from a table (kept in the hop's seg_tab once built), 2 = the per-minibatch kernel
    std::vector<uint8_t> hint_mode;
    std::vector<uint8_t> hint_table_ready; // per hop: seg_tab holds the table for hint_table_C segments
    std::vector<int32_t> hint_table_C;
    // host copies of the per-minibatch offsets (rows, entries, columns: L x 3 x (k+1)), made on demand by
    // bms_result_minibatch and dropped when the result is written again
    std::vector<int64_t> mb_offsets;
    DevBuf mb_edge_tmp;
    Allocator al;               // of the buffers the hop views point to
    // BMS_ASYNC: the call has returned, its kernels may still run
    bool pending = false;
    hipEvent_t done_ev = nullptr;
    int64_t *host_scalars = nullptr; // pinned, 64 values: where the call's sizes and flags arrive
    PendingNodewise deferred;
};

namespace {

void result_release(bms_result *r)
{
    if (r->pending && r->done_ev)
        (void)hipEventSynchronize(r->done_ev); // its kernels still use the buffers
    r->pending = false;
    for (auto &h : r->hops) {
        h.mb_rowoff.release();
        h.row_vertex.release();
        h.rowptr.release();
        h.col.release();
        h.mb_coloff.release();
        h.col_vertex.release();
        h.p_off.release();
        h.p_col.release();
        h.p_cnt.release();
        h.row_self.release();
        h.seg_tab.release();
    }
    r->mb_edge_tmp.release();
    if (r->done_ev)
        (void)hipEventDestroy(r->done_ev);
    r->done_ev = nullptr;
    if (r->host_scalars)
        (void)hipHostFree(r->host_scalars);
    r->host_scalars = nullptr;
    for (auto e : r->event_pool)
        (void)hipEventDestroy(e);
    r->event_pool.clear();
}

// Records one stage between two events when profiling is on.
struct Profiler {
    bms_result *res;
    hipStream_t stream;
    bool on;
    bool main_only = false; // record only the sampler's main kernel stage (BMS_PROFILE_MAIN)
    bool open = false;
    bool skipped = false;   // the running stage is not recorded
    static bool is_main(const char *name)
    {
        return !strcmp(name, "nw_sample") || !strcmp(name, "ldw_accumulate") || !strcmp(name, "ld_accumulate");
    }
    int next_event(hipEvent_t *e)
    {
        while (res->event_pool.size() < res->events_used + 1) {
            hipEvent_t ev;
            HIP_TRY(hipEventCreate(&ev));
            res->event_pool.push_back(ev);
        }
        *e = res->event_pool[res->events_used++];
        return BMS_OK;
    }
    int begin(const char *name, int32_t hop)
    {
        if (!on)
            return BMS_OK;
        if (main_only && !is_main(name)) {
            skipped = true;
            return BMS_OK;
        }
        skipped = false;
        open = true;
        StageTime st{name, hop, nullptr, nullptr, 0.f};
        BMS_TRY(next_event(&st.t0));
        HIP_TRY(hipEventRecord(st.t0, stream));
        res->stages.push_back(st);
        return BMS_OK;
    }
    int end()
    {
        if (!on || !open)
            return BMS_OK;
        open = false;
        StageTime &st = res->stages.back();
        BMS_TRY(next_event(&st.t1));
        HIP_TRY(hipEventRecord(st.t1, stream));
        return BMS_OK;
    }
    // closes the running stage, if any, and opens the next one; one event serves as the end of the first and
    // the start of the second
    int mark(const char *name, int32_t hop)
    {
        if (!on)
            return BMS_OK;
        if (!open || (main_only && !is_main(name))) {
            BMS_TRY(end());
            return begin(name, hop);
        }
        StageTime &prev = res->stages.back();
        BMS_TRY(next_event(&prev.t1));
        HIP_TRY(hipEventRecord(prev.t1, stream));
        StageTime st{name, hop, prev.t1, nullptr, 0.f};
        res->stages.push_back(st);
        return BMS_OK;
    }
    int finish()
    {
        if (!on)
            return BMS_OK;
        for (auto &st : res->stages)
            HIP_TRY(hipEventElapsedTime(&st.ms, st.t0, st.t1));
        return BMS_OK;
    }
};

bool is_device_pointer(const void *p)
{
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError(); // plain host memory reports an error: clear it
        return false;
    }
    return attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged;
}

struct CallCtx {
    bms_csr *csr;
    bms_result *res;
    bool fresh_result;
    hipStream_t stream;
    Launch launch;
    int32_t k, b, L;
    uint64_t seed;
    uint32_t mb_base;
    uint32_t flags;
    int64_t scratch_limit;
    VSet vs;
};

int check_common(const bms_csr *csr, const int32_t *batches, int32_t k, int32_t b, const int32_t *params, int32_t L,
                 const bms_opts *opts, bms_result **out)
{
    if (!csr || csr->tag != kTagCsr)
        return fail(BMS_EINVAL, "csr is not a handle returned by bms_csr_load");
    if (!batches || !params || !out)
        return fail(BMS_EINVAL, "null argument");
    if (k < 1 || b < 1 || L < 1)
        return fail(BMS_EINVAL, "k, b and L must be >= 1 (k=%d b=%d L=%d)", k, b, L);
    if (k > kMaxMinibatches)
        return fail(BMS_EINVAL, "k=%d minibatches per call, at most %d are supported: split the call (mb_base keeps "
                                "the random streams in step)", k, kMaxMinibatches);
    for (int32_t h = 0; h < L; ++h)
        if (params[h] < 1)
            return fail(BMS_EINVAL, "sampling parameter of hop %d is %d, must be >= 1", h, params[h]);
    if (opts) {
        if (opts->flags & ~(BMS_LADIES_SQUARED | BMS_PROFILE | BMS_EXTRACT_BUCKETS | BMS_EXTRACT_BITMAP | BMS_EXTRACT_SORT | BMS_LADIES_DENSE | BMS_PROFILE_MAIN | BMS_UNION_DST | BMS_NODEWISE_REPLACE | BMS_ASYNC | BMS_LADIES_NO_INDEX))
            return fail(BMS_EINVAL, "unknown flag bits 0x%x", opts->flags);
        if (opts->recycle && opts->recycle->tag != kTagResult)
            return fail(BMS_EINVAL, "opts->recycle is not a result handle");
        if (opts->scratch_limit < 0)
            return fail(BMS_EINVAL, "negative scratch_limit");
        if ((opts->alloc == nullptr) != (opts->dealloc == nullptr))
            return fail(BMS_EINVAL, "bms_opts.alloc and bms_opts.dealloc must be given together");
    }
    return BMS_OK;
}

// Sizes the per-minibatch vertex sets, allocates them inside the scratch limit and makes sure
// they start all-zero.
int setup_vset(CallCtx &c)
{
    bms_csr *csr = c.csr;
    VSet &vs = c.vs;
    vs.nl = (csr->n + kLineBits - 1) / kLineBits;
    if (vs.nl < 1)
        vs.nl = 1;
    vs.nw = vs.nl * kLineWords;
    vs.nc = (int32_t)((vs.nl + kChunkLines - 1) / kChunkLines);
    const size_t wbytes = (size_t)c.k * vs.nw * sizeof(uint32_t);
    const size_t pbytes = (size_t)c.k * vs.nl * sizeof(uint32_t);
    const size_t cbytes = ((size_t)c.k * vs.nc + c.k) * sizeof(int64_t);
    if ((int64_t)(wbytes + pbytes + cbytes) > c.scratch_limit)
        return fail(BMS_ENOMEM,
                    "vertex sets for k=%d minibatches over n=%lld vertices need %zu bytes of scratch, limit is %lld: "
                    "raise bms_opts.scratch_limit or sample fewer minibatches per call",
                    c.k, (long long)csr->n, wbytes + pbytes + cbytes, (long long)c.scratch_limit);
    BMS_TRY(csr->vs_words.ensure(wbytes));
    if (csr->vs_words.grew)
        csr->vs_clean = false;
    BMS_TRY(csr->vs_prefix.ensure(pbytes));
    BMS_TRY(csr->vs_chunks.ensure(cbytes));
    vs.words = csr->vs_words.as<uint32_t>();
    vs.line_prefix = csr->vs_prefix.as<uint32_t>();
    vs.chunk_off = csr->vs_chunks.as<int64_t>();
    if (!csr->vs_clean)
        HIP_TRY(hipMemsetAsync(vs.words, 0, csr->vs_words.cap, c.stream));
    csr->vs_clean = false; // dirty until the call completes
    return BMS_OK;
}

int settle_result(bms_result *res);

int begin_call(CallCtx &c, bms_csr *csr, int32_t k, int32_t b, int32_t L, uint64_t seed, const bms_opts *opts)
{
    c.csr = csr;
    c.k = k;
    c.b = b;
    c.L = L;
    c.seed = seed;
    c.stream = opts ? (hipStream_t)opts->stream : nullptr;
    c.mb_base = opts ? (uint32_t)opts->mb_base : 0u;
    c.flags = opts ? opts->flags : 0u;
    c.scratch_limit = (opts && opts->scratch_limit > 0) ? opts->scratch_limit : kDefaultScratchLimit;
    HIP_TRY(hipSetDevice(csr->device));
    BMS_TRY(csr->scan_tmp.ensure(kScanTmpLen * sizeof(int64_t)));
    c.launch = Launch{c.stream, csr->num_cu, csr->scan_tmp.as<int64_t>(), kScanTmpLen};
    c.fresh_result = !(opts && opts->recycle);
    if (c.fresh_result) {
        c.res = new (std::nothrow) bms_result();
        if (!c.res)
            return fail(BMS_ENOMEM, "host allocation failed");
        if (opts) {
            c.res->al.alloc = opts->alloc;
            c.res->al.dealloc = opts->dealloc;
            c.res->al.ctx = opts->alloc_ctx;
        }
    } else {
        c.res = opts->recycle;
        if (c.res->pending)
            (void)settle_result(c.res); // the call before this one: its status belongs to a result nobody looked at
    }
    c.res->k = k;
    c.res->L = L;
    c.res->device = csr->device;
    if ((int32_t)c.res->hops.size() < L)
        c.res->hops.resize(L);
    for (auto &hb : c.res->hops)
        hb.bind(&c.res->al);
    c.res->stages.clear();
    c.res->events_used = 0;
    c.res->mb_offsets.clear();
    if (!csr->host_pinned)
        HIP_TRY(hipHostMalloc((void **)&csr->host_pinned, 64 * sizeof(int64_t), hipHostMallocDefault));
    BMS_TRY(csr->scalars.ensure(64 * sizeof(int64_t)));
    return BMS_OK;
}

int abort_call(CallCtx &c, int rc)
{
    (void)hipStreamSynchronize(c.stream);
    if (c.fresh_result && c.res) {
        result_release(c.res);
        delete c.res;
    } else if (c.res) {
        // a recycled result is left empty: its buffers may have been reallocated while the views still held the old
        // pointers and sizes, so no accessor may hand them out (the handle stays valid for bms_free and for recycling)
        for (auto &h : c.res->hops)
            h.view = bms_hop_view{};
        c.res->L = 0;
        c.res->k = 0;
        c.res->hint_csr = nullptr;
        c.res->mb_offsets.clear();
        c.res->stages.clear();
    }
    c.res = nullptr;
    return rc;
}

// Copies the seeds into hop 0's row_vertex, builds mb_rowoff = i*b and verifies the seeds.
int stage_seeds(CallCtx &c, const int32_t *batches, Profiler &prof, bool use_vset = true)
{
    HopBufs &h0 = c.res->hops[0];
    const size_t nb = (size_t)c.k * c.b;
    BMS_TRY(h0.row_vertex.ensure(nb * sizeof(int32_t)));
    BMS_TRY(h0.mb_rowoff.ensure(((size_t)c.k + 1) * sizeof(int64_t)));
    BMS_TRY(prof.begin("seeds", 0));
    HIP_TRY(hipMemcpyAsync(h0.row_vertex.p, batches, nb * sizeof(int32_t),
                           is_device_pointer(batches) ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice, c.stream));
    launch_iota_offsets(c.launch, h0.mb_rowoff.as<int64_t>(), c.k, c.b);
    int32_t *flag = reinterpret_cast<int32_t *>(c.csr->scalars.as<int64_t>() + 63);
    HIP_TRY(hipMemsetAsync(c.csr->scalars.p, 0, 64 * sizeof(int64_t), c.stream));
    if (use_vset) {
        launch_validate_seeds(c.launch, h0.row_vertex.as<int32_t>(), c.k, c.b, c.csr->n, c.vs, flag);
        launch_clear_seed_bits(c.launch, h0.row_vertex.as<int32_t>(), c.k, c.b, c.csr->n, c.vs);
    } else {
        launch_validate_seeds_sorted(c.launch, h0.row_vertex.as<int32_t>(), c.k, c.b, c.csr->n, flag);
    }
    BMS_TRY(prof.end());
    return BMS_OK;
}

// Device scalars -> pinned host copy, after draining the stream.
int read_scalars(CallCtx &c)
{
    HIP_TRY(hipMemcpyAsync(c.csr->host_pinned, c.csr->scalars.p, 64 * sizeof(int64_t), hipMemcpyDeviceToHost,
                           c.stream));
    HIP_TRY(hipStreamSynchronize(c.stream));
    return BMS_OK;
}

int seed_flag_error(CallCtx &c)
{
    const int32_t flag = (int32_t)(c.csr->host_pinned[63] & 0xFFFFFFFF);
    if (flag & 1)
        return fail(BMS_ERANGE, "a seed vertex lies outside [0, %lld)", (long long)c.csr->n);
    if (flag & 2)
        return fail(BMS_ERANGE, "a seed vertex is repeated inside one minibatch");
    return BMS_OK;
}

// scalar slots: per hop 4 int64: [0] nnz, [1] ncols, [2] pnnz, [3] gathered D ; slot 63 = seed flag
inline int64_t *slot(CallCtx &c, int32_t hop, int which) { return c.csr->scalars.as<int64_t>() + hop * 4 + which; }
inline int64_t host_slot(CallCtx &c, int32_t hop, int which) { return c.csr->host_pinned[hop * 4 + which]; }

constexpr int32_t kMaxHops = 15; // 4 scalar slots per hop in a 64-entry block

// The end of a node-wise call, once its sizes and flags are on the host: deferred seed errors, hops whose EXTRACT
// gave up (*redo), the views' sizes, what the result remembers for the next call of this shape, the stage times.
int finish_nodewise(bms_result *res, const PendingNodewise &pn, const int64_t *host, bool check_seeds, uint32_t *redo)
{
    if (check_seeds) {
        const int32_t flag = (int32_t)(host[63] & 0xFFFFFFFF);
        if (flag & 1)
            return fail(BMS_ERANGE, "a seed vertex lies outside [0, %lld)", (long long)pn.csr->n);
        if (flag & 2)
            return fail(BMS_ERANGE, "a seed vertex is repeated inside one minibatch");
    }
    for (int32_t h = 0; h < pn.L; ++h)
        if (host[h * 4 + 2] & 0xFFFFFFFFLL)
            *redo |= 1u << h;
    if (*redo)
        return BMS_OK; // the call is repeated
    std::vector<int64_t> seen_nnz((size_t)pn.L, 0);
    for (int32_t h = 0; h < pn.L; ++h) {
        bms_hop_view &v = res->hops[h].view;
        v.nnz = host[h * 4 + 0];
        v.ncols = host[h * 4 + 1];
        v.rows = h == 0 ? (int64_t)pn.k * pn.b : host[(h - 1) * 4 + 1];
        seen_nnz[h] = v.nnz + (pn.union_dst ? v.rows : 0); // the entries EXTRACT worked on
    }
    res->hint_csr = pn.csr;
    res->hint_shape = pn.shape;
    res->hint_nnz = seen_nnz;
    res->hint_mode = pn.mode;
    res->hint_table_C = pn.table_built;
    res->hint_table_ready.assign((size_t)pn.L, 0);
    for (int32_t h = 0; h < pn.L; ++h)
        res->hint_table_ready[h] = pn.table_built[h] > 0 ? 1 : 0;
    for (auto &st : res->stages)
        HIP_TRY(hipEventElapsedTime(&st.ms, st.t0, st.t1));
    return BMS_OK;
}

void empty_result(bms_result *r, bool keep_hints)
{
    for (auto &h : r->hops)
        h.view = bms_hop_view{};
    r->L = 0;
    r->k = 0;
    if (!keep_hints)
        r->hint_csr = nullptr;
    r->mb_offsets.clear();
}

// First look at the result of a BMS_ASYNC call: waits for it and returns what the call would have returned.
int settle_result(bms_result *res)
{
    if (!res->pending)
        return BMS_OK;
    res->pending = false;
    HIP_TRY(hipSetDevice(res->device));
    HIP_TRY(hipEventSynchronize(res->done_ev));
    uint32_t redo = 0;
    const int rc = finish_nodewise(res, res->deferred, res->host_scalars, true, &redo);
    if (rc != BMS_OK) {
        empty_result(res, false);
        return rc;
    }
    if (redo) {
        // the next call of this shape starts with the kernel path after the one that gave up
        if ((int32_t)res->hint_mode.size() == res->deferred.L)
            for (int32_t h = 0; h < res->deferred.L; ++h)
                if ((redo >> h) & 1u)
                    res->hint_mode[h] = (uint8_t)std::min<int>(res->hint_mode[h] + 1, 2);
        empty_result(res, true);
        return fail(BMS_EAGAIN, "the asynchronous call's EXTRACT gave up on this input (sampled ids crowd a narrow id range): "
                                "repeat the call");
    }
    return BMS_OK;
}

// what a recycled result remembers a call by
std::vector<int32_t> nodewise_shape(const CallCtx &c, const int32_t *fanouts)
{
    std::vector<int32_t> shape{c.k, c.b, ((c.flags & BMS_UNION_DST) ? 1 : 0) | ((c.flags & BMS_NODEWISE_REPLACE) ? 2 : 0)};
    shape.insert(shape.end(), fanouts, fanouts + c.L);
    return shape;
}

// One attempt.  *redo receives the hops (bits) whose EXTRACT by id-range segments gave up (ids crowded into a narrow
// range): the result is then incomplete and the caller repeats the call with those hops moved to the next mode.
int sample_nodewise_once(CallCtx &c, const int32_t *batches, const int32_t *fanouts, const std::vector<uint8_t> &mode,
                         uint32_t *redo)
{
    bms_csr *csr = c.csr;
    Profiler prof{c.res, c.stream, (c.flags & (BMS_PROFILE | BMS_PROFILE_MAIN)) != 0, (c.flags & BMS_PROFILE) == 0};
    // EXTRACT strategy: LDS sorts of id-range segments (with the per-minibatch bin kernel as the
    // fallback for crowded id ranges) whenever the bin table of that fallback fits in LDS; the
    // per-minibatch bitmaps over [0,n) in HBM otherwise.
    const int64_t nbuckets = std::max<int64_t>((csr->n + (1LL << kBucketBits) - 1) >> kBucketBits, 1);
    bool buckets = true;
    bool seg_sort = true; // with buckets: sort id-range segments in LDS, per-minibatch kernel as fallback
    if (c.flags & BMS_EXTRACT_SORT)
        buckets = true;
    if (c.flags & BMS_EXTRACT_BUCKETS) {
        buckets = true;
        seg_sort = false;
    }
    if (c.flags & BMS_EXTRACT_BITMAP)
        buckets = false;
    if (nbuckets > kMaxBuckets)
        buckets = false;
    const bool seeds_by_sort = buckets && c.b <= kMaxSortedSeeds;
    if (!buckets || !seeds_by_sort)
        BMS_TRY(setup_vset(c));
    BMS_TRY(stage_seeds(c, batches, prof, !seeds_by_sort));
    if (buckets) {
        BMS_TRY(csr->dd_edgeoff.ensure(((size_t)c.k + 1) * sizeof(int64_t)));
        BMS_TRY(csr->dd_count.ensure((size_t)c.k * sizeof(int64_t)));
        BMS_TRY(csr->dd_done.ensure(256));
        HIP_TRY(hipMemsetAsync(csr->dd_done.p, 0, 256, c.stream));
    }
    std::vector<int32_t> table_built((size_t)c.L, 0); // per hop: segments of the table in use (0: none)
    int32_t table_pending = -1;
    bool tiles_planned = false;        // the hop's row tiles were written by the hop before it
    bool counters_zero = csr->segcnt_clean; // the segment counters are all zero between hops: the kernels clear what they
    csr->segcnt_clean = false;              // read; a fresh buffer, or one an interrupted call left behind, is cleared here

    int64_t rows_bound = (int64_t)c.k * c.b;
    const int32_t *row_vertex = c.res->hops[0].row_vertex.as<int32_t>();
    const int64_t *mb_rowoff = c.res->hops[0].mb_rowoff.as<int64_t>();
    BMS_TRY(csr->mb_tileoff.ensure(((size_t)c.k + 2) * sizeof(int64_t)));

    // Steady state: a recycled result that remembers the sizes of the same call shape lets every hop
    // be enqueued without a host round trip.  Buffers are then sized by the upper bound
    // rows * min(s, max degree) (always enough), tuning parameters by the remembered sizes.
    const bool union_dst = (c.flags & BMS_UNION_DST) != 0;
    const bool replace = (c.flags & BMS_NODEWISE_REPLACE) != 0;
    const std::vector<int32_t> shape = nodewise_shape(c, fanouts);
    bool no_wait = buckets && !c.fresh_result && c.res->hint_csr == csr && c.res->hint_shape == shape &&
                   (int32_t)c.res->hint_nnz.size() == c.L;
    if (no_wait) {
        double bound = (double)rows_bound, total = 0.0;
        for (int32_t h = 0; h < c.L; ++h) {
            bound *= (double)std::min<int64_t>(fanouts[h], std::max<int64_t>(csr->max_degree, 1)) + (union_dst ? 1.0 : 0.0);
            total += bound * 40.0; // bytes of result + scratch per sampled edge, generously
            bound = std::min(bound, (double)c.k * (double)csr->n);
        }
        no_wait = total < (double)c.scratch_limit;
    }

    for (int32_t h = 0; h < c.L; ++h) {
        HopBufs &hb = c.res->hops[h];
        const int64_t tiles_bound = rows_bound / kRowTile + c.k;
        BMS_TRY(csr->row_beg.ensure((size_t)std::max<int64_t>(rows_bound, 1) * sizeof(int64_t)));
        BMS_TRY(csr->row_deg.ensure((size_t)std::max<int64_t>(rows_bound, 1) * sizeof(int32_t)));
        BMS_TRY(csr->tile_off.ensure((size_t)(tiles_bound + 2) * sizeof(int64_t)));
        BMS_TRY(hb.rowptr.ensure((size_t)(rows_bound + 1) * sizeof(int64_t)));
        BMS_TRY(hb.mb_coloff.ensure(((size_t)c.k + 1) * sizeof(int64_t)));
        if (union_dst) {
            BMS_TRY(csr->un_rowptr.ensure((size_t)(rows_bound + 1) * sizeof(int64_t)));
            BMS_TRY(hb.row_self.ensure((size_t)std::max<int64_t>(rows_bound, 1) * sizeof(int32_t)));
        }

        NwHop a{};
        a.A_rowptr = csr->rowptr;
        a.A_col = csr->col;
        a.n = csr->n;
        a.k = c.k;
        a.s = fanouts[h];
        a.hopkey = hop_key(c.seed, h);
        a.mb_base = c.mb_base;
        a.row_vertex = row_vertex;
        a.mb_rowoff = mb_rowoff;
        a.mb_tileoff = csr->mb_tileoff.as<int64_t>();
        a.row_beg = csr->row_beg.as<int64_t>();
        a.row_deg = csr->row_deg.as<int32_t>();
        a.tile_off = csr->tile_off.as<int64_t>();
        // with BMS_UNION_DST the hop is built with one more entry per row (the row's own vertex) in scratch
        // and moved to the result's arrays without it at the end of the hop
        a.out_rowptr = union_dst ? csr->un_rowptr.as<int64_t>() : hb.rowptr.as<int64_t>();
        a.rows_bound = rows_bound;
        a.self_entry = union_dst ? 1 : 0;
        a.replace = replace ? 1 : 0;
        if (replace && a.s > 32) {
            BMS_TRY(csr->row_cnt.ensure((size_t)std::max<int64_t>(rows_bound, 1) * sizeof(int32_t)));
            a.row_cnt = csr->row_cnt.as<int32_t>();
        }

        BMS_TRY(prof.begin("nw_rows", h));
        if (!tiles_planned)
            launch_plan_tiles(c.launch, mb_rowoff, c.k, kRowTile, a.mb_tileoff, a.mb_tileoff + c.k + 1);
        tiles_planned = false;
        launch_nw_rows(c.launch, a);
        BMS_TRY(prof.end());
        BMS_TRY(prof.begin("scan_tiles", h));
        launch_scan_i64(c.launch, a.tile_off, a.mb_tileoff + c.k, slot(c, h, 0), a.out_rowptr, mb_rowoff + c.k,
                        rows_bound / kRowTile + c.k);
        BMS_TRY(prof.end());

        // nnz sizes the column buffers: read back (the only host round trip of the hop), or in the
        // steady state bounded from above; nnz_tune only picks tuning parameters
        int64_t nnz, nnz_tune;
        if (no_wait) { // with BMS_UNION_DST nnz counts the rows' own entries too, until the hop's last step
            nnz = rows_bound * (std::min<int64_t>(fanouts[h], std::max<int64_t>(csr->max_degree, 1)) + a.self_entry);
            nnz_tune = std::max<int64_t>(c.res->hint_nnz[h], 1);
        } else {
            BMS_TRY(read_scalars(c));
            if (h == 0)
                BMS_TRY(seed_flag_error(c));
            nnz = nnz_tune = host_slot(c, h, 0);
        }
        const int64_t ncols_bound = std::min<int64_t>(nnz, (int64_t)c.k * csr->n);
        BMS_TRY(hb.col.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(int32_t)));
        BMS_TRY(hb.col_vertex.ensure((size_t)std::max<int64_t>(ncols_bound, 1) * sizeof(int32_t)));
        if (union_dst)
            BMS_TRY(csr->un_col.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(int32_t)));
        a.out_col = union_dst ? csr->un_col.as<int32_t>() : hb.col.as<int32_t>();

        DedupArgs d{};
        bool counted = false;
        if (buckets) {
            BMS_TRY(csr->dd_pairs.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(uint64_t)));
            BMS_TRY(csr->dd_utmp.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(uint64_t)));
            // segments = id ranges of 2^cshift ids holding 1500..3000 sampled ids each on average (one workgroup ranks
            // up to 4096 in LDS; the longer a segment, the longer the runs the cut appends to it per tile),
            // at most kMaxSegments of them
            int32_t C = 0, cshift = 0, by_bitmap = 0, fshift = 0, wbits_max = 0, target_per_mb = 0;
            const bool by_table = mode[h] == 1;
            if (seg_sort && mode[h] < 2) {
                const double per_mb = (double)nnz_tune / c.k + 1.0;
                // ids dense enough in [0, n) that a pass over a bitmap of a segment's id range costs less than sorting
                // its ids: segments as wide as the bitmap kernel takes, as long as they hold well under 2^16 ids
                by_bitmap = (double)csr->n <= kBitmapIdsPerEntry * per_mb ? 1 : 0;
                const double target = by_bitmap ? 16384.0 : 3000.0;
                const int32_t most = by_bitmap ? kMaxBitmapShift : 31;
                cshift = 0;
                while (cshift < most && (double)(2LL << cshift) * per_mb <= target * (double)csr->n)
                    ++cshift;
                while (((csr->n + (1LL << cshift) - 1) >> cshift) > kMaxSegments)
                    ++cshift;
                if (cshift > kMaxBitmapShift)
                    by_bitmap = 0;
                C = (int32_t)std::max<int64_t>((csr->n + (1LL << cshift) - 1) >> cshift, 1);
                wbits_max = std::min(cshift, kMaxBitmapShift);
                if (by_table) {
                    // segments of unequal width: cells of 2^fshift ids (at most kMaxCells of them) dealt to segments of
                    // about 2/3 of what the ranking kernels take; room for twice the expected number of segments
                    while (((csr->n + (1LL << fshift) - 1) >> fshift) > kMaxCells)
                        ++fshift;
                    target_per_mb = by_bitmap ? 16384 : 2500;
                    wbits_max = by_bitmap ? std::max(cshift, fshift) : kMaxBitmapShift;
                    const int64_t cells = std::max<int64_t>((csr->n + (1LL << fshift) - 1) >> fshift, 1);
                    const int64_t forced = by_bitmap ? (cells >> std::max(wbits_max - fshift, 0)) + 2 : 3;
                    C = (int32_t)std::min<int64_t>(kMaxSegments, (int64_t)(2.0 * per_mb / target_per_mb) + forced + 8);
                    if (!c.fresh_result && h < (int32_t)c.res->hint_table_ready.size() && c.res->hint_table_ready[h] &&
                        no_wait)
                        C = c.res->hint_table_C[h]; // the table at hand was built for this many
                }
                // few sampled edges per minibatch: the single per-minibatch kernel beats the chain of
                // chip-wide kernels, whose launches would dominate (unless that path was asked for)
                if (per_mb <= 4096.0 && !(c.flags & BMS_EXTRACT_SORT))
                    C = 0;
            }
            const size_t stride = (size_t)std::max<int64_t>(nbuckets, C);
            const size_t kC = (size_t)c.k * (size_t)C;
            const int64_t xtiles = nnz / kCutTile + c.k; // tiles of the cut
            BMS_TRY(csr->dd_uniq.ensure((size_t)c.k * stride * sizeof(uint32_t)));
            BMS_TRY(csr->dd_seg.ensure((3 * kC + (size_t)c.k + 16) * sizeof(uint32_t)));
            BMS_TRY(csr->dd_segcnt.ensure(std::max<size_t>(kC, 1) * sizeof(uint32_t)));
            if (csr->dd_segcnt.grew || !counters_zero) {
                HIP_TRY(hipMemsetAsync(csr->dd_segcnt.p, 0, csr->dd_segcnt.cap, c.stream));
                counters_zero = true;
            }
            BMS_TRY(csr->dd_runs.ensure(2 * (size_t)xtiles * (size_t)std::max(C, 1) * sizeof(uint32_t)));
            BMS_TRY(csr->dd_tileoff.ensure(3 * ((size_t)c.k + 1) * sizeof(int64_t)));
            d.k = c.k;
            d.nbuckets = (int32_t)nbuckets;
            d.mb_edgeoff = csr->dd_edgeoff.as<int64_t>();
            d.col = a.out_col;
            d.pairs = csr->dd_pairs.as<uint64_t>();
            d.utmp = csr->dd_utmp.as<uint64_t>();
            d.bin_base = csr->dd_uniq.as<uint32_t>();
            BMS_TRY(csr->dd_back.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(uint64_t)));
            BMS_TRY(csr->dd_cursor.ensure((size_t)(nnz / kDedupPlaceTile + c.k + 1) * sizeof(uint32_t)));
            d.back = csr->dd_back.as<uint64_t>();
            d.split_tileoff = csr->dd_tileoff.as<int64_t>();
            d.place_tileoff = csr->dd_tileoff.as<int64_t>() + c.k + 1;
            d.place_cursor = csr->dd_cursor.as<uint32_t>();
            d.stride = (int32_t)stride;
            d.C = C;
            d.cshift = cshift;
            d.by_bitmap = by_bitmap;
            d.wbits_max = wbits_max;
            bool build_table = false;
            if (C > 0 && by_table) {
                BMS_TRY(hb.seg_tab.ensure((size_t)(kMaxCells + 2) * sizeof(uint16_t) + ((size_t)kMaxSegments + 2) * sizeof(uint32_t)));
                BMS_TRY(csr->dd_hist.ensure(((size_t)kMaxCells + 2) * sizeof(uint32_t)));
                d.tab = hb.seg_tab.as<uint16_t>();
                d.seg_first = reinterpret_cast<const uint32_t *>(hb.seg_tab.as<uint16_t>() + kMaxCells + 2);
                d.fshift = fshift;
                const bool ready = no_wait && h < (int32_t)c.res->hint_table_ready.size() && c.res->hint_table_ready[h] &&
                                   c.res->hint_table_C[h] == C && !hb.seg_tab.grew;
                build_table = !ready;
            }
            d.big_tileoff = csr->dd_tileoff.as<int64_t>() + 2 * (c.k + 1);
            // flag and list counter of the hop: two 32-bit words of a scalar slot, zeroed with the slots at the start of
            // the call and read back with the sizes at its end
            d.fallback = C ? reinterpret_cast<int32_t *>(slot(c, h, 2)) : nullptr;
            d.big_count = reinterpret_cast<uint32_t *>(slot(c, h, 2)) + 1;
            d.seg_cnt = csr->dd_segcnt.as<uint32_t>();
            d.seg_off = csr->dd_seg.as<uint32_t>();
            d.seg_cursor = d.seg_off + kC + c.k;
            d.big_list = d.seg_cursor + kC;
            // the segment path keeps the ids grouped by segment and the per-position words in the first buffer,
            // the distinct ids and the 16-bit ranks in the second (the per-minibatch path uses both as 8-byte entries)
            d.ids_seg = csr->dd_pairs.as<uint32_t>();
            d.loc = d.ids_seg + std::max<int64_t>(nnz, 1);
            d.uids = csr->dd_utmp.as<uint32_t>();
            d.ranks = reinterpret_cast<uint16_t *>(d.uids + std::max<int64_t>(nnz, 1));
            d.run_gpos = csr->dd_runs.as<uint32_t>();
            d.run_cnt = d.run_gpos + (size_t)xtiles * (size_t)std::max(C, 1);
            d.mb_count = csr->dd_count.as<int64_t>();
            if (C > 0 && !build_table) { // the sampling kernel counts the ids per segment while it has them in LDS, when it can
                a.seg_cnt = d.seg_cnt;
                a.seg_C = C;
                a.seg_shift = by_table ? fshift : cshift;
                a.seg_tab = d.tab;
            }
            table_built[h] = (C > 0 && by_table) ? C : 0;
            if (build_table)
                table_pending = h;
        }
        BMS_TRY(prof.begin("nw_sample", h));
        counted = launch_nw_sample(c.launch, a, c.vs, !buckets);
        BMS_TRY(prof.end());
        if (table_pending == h) { // the table of this hop's segments, from a sample of the ids just staged
            BMS_TRY(prof.begin("dd_table", h));
            launch_nw_dedup_table(c.launch, a.out_col, slot(c, h, 0), nnz, csr->n, c.k, d.fshift, d.C,
                                  d.by_bitmap ? 16384 : 2500, d.by_bitmap ? d.wbits_max : 31, csr->dd_hist.as<uint32_t>(),
                                  const_cast<uint16_t *>(d.tab), const_cast<uint32_t *>(d.seg_first));
            BMS_TRY(prof.end());
        }
        if (buckets) {
            const StageMark mark = [&](const char *name) { (void)prof.mark(name, h); };
            if (d.C > 0) {
                launch_nw_extract_segments(c.launch, d, a.out_rowptr, mb_rowoff, hb.mb_coloff.as<int64_t>(),
                                           hb.col_vertex.as<int32_t>(), slot(c, h, 1), csr->mb_tileoff.as<int64_t>(),
                                           csr->dd_done.as<uint32_t>(), nnz, counted, mark);
                tiles_planned = true;
            } else if (launch_nw_dedup_bucket(c.launch, d, a.out_rowptr, mb_rowoff, hb.mb_coloff.as<int64_t>(),
                                              hb.col_vertex.as<int32_t>(), slot(c, h, 1), nnz, mark) != 0) {
                return fail(BMS_EHIP, "launch of the bucket EXTRACT kernel was refused");
            }
            BMS_TRY(prof.end());
        } else {
            BMS_TRY(prof.begin("vset_rank", h));
            launch_vset_rank(c.launch, c.vs, c.k, hb.mb_coloff.as<int64_t>(), hb.col_vertex.as<int32_t>(),
                             slot(c, h, 1));
            BMS_TRY(prof.end());
            BMS_TRY(prof.begin("nw_relabel", h));
            launch_nw_relabel(c.launch, a, c.vs);
            BMS_TRY(prof.end());
            BMS_TRY(prof.begin("vset_clear", h));
            launch_vset_clear(c.launch, c.vs, c.k, hb.mb_coloff.as<int64_t>(), hb.col_vertex.as<int32_t>(),
                              ncols_bound);
            BMS_TRY(prof.end());
        }

        if (union_dst) {
            BMS_TRY(prof.begin("nw_strip_self", h));
            launch_nw_strip_self(c.launch, a.out_rowptr, a.out_col, mb_rowoff + c.k, rows_bound, hb.rowptr.as<int64_t>(),
                                 hb.col.as<int32_t>(), hb.row_self.as<int32_t>(), slot(c, h, 0));
            BMS_TRY(prof.end());
        }

        hb.view = bms_hop_view{};
        hb.view.nnz = nnz;
        hb.view.row_self = union_dst ? hb.row_self.as<int32_t>() : nullptr;
        hb.view.mb_rowoff = mb_rowoff;
        hb.view.row_vertex = row_vertex;
        hb.view.rowptr = hb.rowptr.as<int64_t>();
        hb.view.col = hb.col.as<int32_t>();
        hb.view.mb_coloff = hb.mb_coloff.as<int64_t>();
        hb.view.col_vertex = hb.col_vertex.as<int32_t>();

        row_vertex = hb.col_vertex.as<int32_t>();
        mb_rowoff = hb.mb_coloff.as<int64_t>();
        rows_bound = ncols_bound;
    }
    csr->segcnt_clean = true; // every hop's kernels are enqueued: they leave the counters at zero again
    PendingNodewise pn;
    pn.csr = csr;
    pn.k = c.k;
    pn.b = c.b;
    pn.L = c.L;
    pn.union_dst = union_dst;
    pn.shape = shape;
    pn.mode = mode;
    pn.table_built = table_built;
    if ((c.flags & BMS_ASYNC) && no_wait && seeds_by_sort) {
        // steady state, asynchronous: the sizes and flags travel to pinned memory of the result behind the kernels,
        // an event marks their arrival, and the first look at the result does what follows below
        if (!c.res->host_scalars)
            HIP_TRY(hipHostMalloc((void **)&c.res->host_scalars, 64 * sizeof(int64_t), hipHostMallocDefault));
        if (!c.res->done_ev)
            HIP_TRY(hipEventCreateWithFlags(&c.res->done_ev, hipEventDisableTiming));
        HIP_TRY(hipMemcpyAsync(c.res->host_scalars, csr->scalars.p, 64 * sizeof(int64_t), hipMemcpyDeviceToHost, c.stream));
        HIP_TRY(hipEventRecord(c.res->done_ev, c.stream));
        c.res->deferred = std::move(pn);
        c.res->pending = true;
        return BMS_OK;
    }
    BMS_TRY(read_scalars(c));
    BMS_TRY(finish_nodewise(c.res, pn, csr->host_pinned, no_wait, redo));
    if (!*redo && (!buckets || !seeds_by_sort))
        csr->vs_clean = true;
    return BMS_OK;
}

int sample_nodewise_impl(CallCtx &c, const int32_t *batches, const int32_t *fanouts)
{
    // hops that gave up on a kernel path in an earlier call of this shape start with the path that worked then
    std::vector<uint8_t> mode((size_t)c.L, 0);
    if (!c.fresh_result && c.res->hint_csr == c.csr && c.res->hint_shape == nodewise_shape(c, fanouts) &&
        (int32_t)c.res->hint_mode.size() == c.L)
        mode = c.res->hint_mode;
    for (int32_t attempt = 0; attempt <= 2 * c.L; ++attempt) {
        uint32_t redo = 0;
        c.res->attempts = attempt + 1;
        BMS_TRY(sample_nodewise_once(c, batches, fanouts, mode, &redo));
        if (!redo)
            return BMS_OK;
        for (int32_t h = 0; h < c.L; ++h)
            if ((redo >> h) & 1u)
                mode[h] = (uint8_t)std::min<int>(mode[h] + 1, 2);
        c.res->stages.clear();
        c.res->events_used = 0;
    }
    return fail(BMS_EHIP, "EXTRACT did not settle on a kernel path");
}

// LADIES with the column counts of P accumulated in LDS, one window of 2^16 vertex ids at a time.
bool ladies_windows_apply(const CallCtx &c, const int32_t *s_per_layer)
{
    if (c.flags & BMS_LADIES_DENSE)
        return false;
    if (c.b > kMaxSortedSeeds || c.b > kMaxWinRows)
        return false;
    for (int32_t h = 0; h < c.L; ++h)
        if (s_per_layer[h] > kMaxWinSampled)
            return false;
    return true;
}

// The window boundaries of every vertex's adjacency list, once per graph: the boundary pass of a hop whose one
// minibatch has all n vertices as rows.  Built when the lists take no more room than twice the adjacency's
// column array and a quarter of the scratch limit; a call that cannot build it computes its rows' lists itself.
int build_window_index(CallCtx &c, int32_t nwin)
{
    bms_csr *csr = c.csr;
    csr->lw_index_tried = true;
    const size_t ibytes = (size_t)csr->n * (size_t)(nwin + 1) * sizeof(uint32_t);
    if (csr->n == 0 || csr->nnz == 0 || ibytes > 2 * (size_t)csr->nnz * sizeof(int32_t) ||
        (int64_t)ibytes > c.scratch_limit / 4)
        return BMS_OK;
    if (csr->lw_index.ensure(ibytes) != BMS_OK) {
        (void)hipGetLastError(); // no room: the hops go without
        return BMS_OK;
    }
    LwHop g{};
    g.A_rowptr = csr->rowptr;
    g.A_col = csr->col;
    g.n = csr->n;
    g.k = 1;
    g.nwin = nwin;
    g.tile = kLwTileMax;
    g.tiles_bound = csr->nnz / g.tile + 1;
    BMS_TRY(csr->lw_tiles.ensure((size_t)g.tiles_bound * (sizeof(int64_t) + sizeof(uint32_t)) + 64));
    int64_t *small = csr->lw_count.as<int64_t>(); // at least 8 words
    launch_iota_offsets(c.launch, small, 1, csr->n); // the one minibatch: rows 0 .. n
    g.mb_rowoff = small;
    g.mb_goff = small + 2;
    g.mb_gtileoff = small + 4;
    g.rows_bound = csr->n;
    g.gather_off = csr->rowptr; // the gathered order of all rows is the adjacency itself
    g.row_beg = csr->rowptr;
    g.tile_row = csr->lw_tiles.as<int64_t>();
    g.bounds = csr->lw_index.as<uint32_t>();
    HIP_TRY(hipMemsetAsync(g.bounds, 0, ibytes, c.stream)); // vertices without neighbours get no list
    launch_ldw_index(c.launch, g);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize(c.stream)); // later calls may come on other streams
    csr->lw_index_ready = true;
    return BMS_OK;
}

// what a layer-wise call is remembered by: a later call of the same shape on a recycled result sizes its buffers
// from what this one needed (node-wise shapes have 0..3 in the third place)
std::vector<int32_t> ladies_shape(const CallCtx &c, const int32_t *s_per_layer)
{
    std::vector<int32_t> shape{c.k, c.b, 16 | ((c.flags & BMS_LADIES_SQUARED) ? 1 : 0)};
    shape.insert(shape.end(), s_per_layer, s_per_layer + c.L);
    return shape;
}

// room provided for a size that an earlier call of the same shape put at `seen`
inline int64_t with_margin(int64_t seen) { return seen + seen / 4 + 65536; }

// One attempt.  may_skip_waits: the sizes of a recycled result's last call of this shape may stand in for
// read-backs.  *redo: they did not suffice (the device flag went up): the result is incomplete, repeat without.
int sample_ladies_windows_once(CallCtx &c, const int32_t *batches, const int32_t *s_per_layer, bool may_skip_waits,
                               bool *redo)
{
    bms_csr *csr = c.csr;
    *redo = false;
    Profiler prof{c.res, c.stream, (c.flags & (BMS_PROFILE | BMS_PROFILE_MAIN)) != 0, (c.flags & BMS_PROFILE) == 0};
    const int64_t n1 = std::max<int64_t>(csr->n, 1);
    const int32_t nwin = (int32_t)((n1 + (1LL << kWinShift) - 1) >> kWinShift);
    const size_t nw = (size_t)c.k * nwin;
    BMS_TRY(csr->lw_win.ensure(nw * (2 * sizeof(uint32_t) + 3 * sizeof(int64_t)) + 64));
    BMS_TRY(csr->lw_parts.ensure(nw * kWinParts * (2 * sizeof(uint32_t) + 3 * sizeof(uint64_t))));
    BMS_TRY(csr->lw_count.ensure((4 * (size_t)c.k + 4) * sizeof(int64_t)));
    if (!csr->lw_index_tried && !(c.flags & BMS_LADIES_NO_INDEX))
        BMS_TRY(build_window_index(c, nwin));
    const uint32_t *index = csr->lw_index_ready && !(c.flags & BMS_LADIES_NO_INDEX) ? csr->lw_index.as<uint32_t>() : nullptr;
    const size_t blists = index ? 1 : 2; // boundary lists held per hop: window-major only, or row-major as well
    BMS_TRY(stage_seeds(c, batches, prof, false));

    int64_t rows_bound = (int64_t)c.k * c.b;
    const int32_t *row_vertex = c.res->hops[0].row_vertex.as<int32_t>();
    const int64_t *mb_rowoff = c.res->hops[0].mb_rowoff.as<int64_t>();

    // Steady state: a recycled result that remembers what the same call shape needed lets every hop be enqueued
    // without a host round trip; the kernels check the sizes they find against what was provided (LwHop::giveup)
    const std::vector<int32_t> shape = ladies_shape(c, s_per_layer);
    const bool no_wait = may_skip_waits && !c.fresh_result && c.res->hint_csr == csr && c.res->hint_shape == shape &&
                         (int32_t)c.res->hint_gathered.size() == c.L && (int32_t)c.res->hint_pnnz.size() == c.L &&
                         (int32_t)c.res->hint_nnz.size() == c.L;
    int32_t *giveup = reinterpret_cast<int32_t *>(csr->scalars.as<int64_t>() + 60);

    for (int32_t h = 0; h < c.L; ++h) {
        HopBufs &hb = c.res->hops[h];
        const int32_t s = s_per_layer[h];
        const int64_t ncols_bound = (int64_t)c.k * std::min<int64_t>(s, n1);
        const size_t bbytes = (size_t)(nwin + 1) * (size_t)rows_bound * sizeof(uint32_t);
        if ((int64_t)(blists * bbytes) > c.scratch_limit)
            return fail(BMS_ENOMEM, "window boundaries of %lld rows need %zu bytes of scratch, limit is %lld: raise "
                                    "bms_opts.scratch_limit or sample fewer minibatches per call",
                        (long long)rows_bound, blists * bbytes, (long long)c.scratch_limit);
        BMS_TRY(csr->row_beg.ensure((size_t)rows_bound * sizeof(int64_t)));
        BMS_TRY(csr->ld_gather_off.ensure((size_t)(rows_bound + 1) * sizeof(int64_t)));
        BMS_TRY(csr->ld_row_mb.ensure((size_t)rows_bound * sizeof(int32_t)));
        BMS_TRY(csr->lw_bounds.ensure(blists * bbytes));
        BMS_TRY(csr->lw_sel.ensure((size_t)c.k * (size_t)s * sizeof(int32_t)));
        BMS_TRY(hb.rowptr.ensure((size_t)(rows_bound + 1) * sizeof(int64_t)));
        BMS_TRY(hb.mb_coloff.ensure(((size_t)c.k + 1) * sizeof(int64_t)));
        BMS_TRY(hb.col_vertex.ensure((size_t)ncols_bound * sizeof(int32_t)));
        BMS_TRY(hb.p_off.ensure(((size_t)c.k + 1) * sizeof(int64_t)));

        LdHop a{};
        a.A_rowptr = csr->rowptr;
        a.A_col = csr->col;
        a.n = csr->n;
        a.k = c.k;
        a.s = s;
        a.row_vertex = row_vertex;
        a.mb_rowoff = mb_rowoff;
        a.rows_bound = rows_bound;
        a.row_beg = csr->row_beg.as<int64_t>();
        a.gather_off = csr->ld_gather_off.as<int64_t>();
        a.row_mb = csr->ld_row_mb.as<int32_t>();
        a.gather_tiles = csr->scalars.as<int64_t>() + 62;
        a.out_rowptr = hb.rowptr.as<int64_t>();

        LwHop w{};
        w.A_rowptr = csr->rowptr;
        w.A_col = csr->col;
        w.n = csr->n;
        w.k = c.k;
        w.s = s;
        w.squared = (c.flags & BMS_LADIES_SQUARED) ? 1 : 0;
        w.hopkey = hop_key(c.seed, h);
        w.mb_base = c.mb_base;
        w.row_vertex = row_vertex;
        w.mb_rowoff = mb_rowoff;
        w.rows_bound = rows_bound;
        w.row_beg = a.row_beg;
        w.gather_off = a.gather_off;
        w.nwin = nwin;
        w.index = index;
        w.bounds = index ? nullptr : csr->lw_bounds.as<uint32_t>() + (size_t)(nwin + 1) * (size_t)rows_bound;
        w.bounds_t = csr->lw_bounds.as<uint32_t>();
        w.win_wt = csr->lw_win.as<uint64_t>();
        w.win_woff = w.win_wt + nw;
        w.win_poff = reinterpret_cast<int64_t *>(w.win_woff + nw);
        w.win_cnt = reinterpret_cast<uint32_t *>(w.win_poff + nw);
        w.win_added = w.win_cnt + nw;
        w.part_woff = csr->lw_parts.as<uint64_t>();
        w.part_wt = w.part_woff + nw * kWinParts;
        w.part_base = reinterpret_cast<int64_t *>(w.part_wt + nw * kWinParts);
        w.part_off = reinterpret_cast<uint32_t *>(w.part_base + nw * kWinParts);
        w.part_cnt = w.part_off + nw * kWinParts;
        w.cursor = reinterpret_cast<unsigned long long *>(csr->scalars.as<int64_t>() + 61);
        w.mb_count = csr->lw_count.as<int64_t>();
        w.mb_goff = w.mb_count + c.k + 1;
        w.mb_gtileoff = w.mb_goff + c.k + 1;
        w.tile_queue = reinterpret_cast<unsigned long long *>(w.mb_gtileoff + c.k + 1);
        w.row_mb = a.row_mb;
        w.p_off = hb.p_off.as<int64_t>();
        w.sel_tmp = csr->lw_sel.as<int32_t>();
        w.mb_coloff = hb.mb_coloff.as<int64_t>();
        w.col_vertex = hb.col_vertex.as<int32_t>();
        w.out_rowptr = hb.rowptr.as<int64_t>();

        // P = Q A
        BMS_TRY(prof.begin("ld_rows", h));
        launch_ld_rows(c.launch, a, slot(c, h, 3));
        BMS_TRY(prof.end());
        int64_t D; // gathered neighbours: sizes the staging of P and of the kept neighbours
        if (no_wait) {
            D = with_margin(c.res->hint_gathered[h]);
        } else {
            BMS_TRY(read_scalars(c));
            if (h == 0)
                BMS_TRY(seed_flag_error(c));
            D = host_slot(c, h, 3);
        }
        w.giveup = giveup;
        w.gathered_cap = D;
        // every part of a window claims room for as many columns as it has ids, or as the window has neighbours
        const int64_t tmp_cap = std::max<int64_t>(std::min<int64_t>(kWinParts * D, (int64_t)nw << kWinShift), 1);
        const size_t tbytes = (size_t)tmp_cap * 4 + (size_t)std::max<int64_t>(D, 1) * 4;
        if (no_wait && (int64_t)(tbytes + blists * bbytes) > c.scratch_limit) {
            *redo = true; // the margin does not fit the limit; the exact sizes may
            return BMS_OK;
        }
        if ((int64_t)(tbytes + blists * bbytes) > c.scratch_limit)
            return fail(BMS_ENOMEM, "%lld gathered neighbours need %zu bytes of scratch, limit is %lld: raise "
                                    "bms_opts.scratch_limit or sample fewer minibatches per call",
                        (long long)D, tbytes + blists * bbytes, (long long)c.scratch_limit);
        BMS_TRY(csr->lw_tmpcol.ensure((size_t)tmp_cap * sizeof(int32_t)));
        BMS_TRY(csr->lw_xtmp.ensure((size_t)std::max<int64_t>(D, 1) * sizeof(int32_t)));
        w.tmp_ent = csr->lw_tmpcol.as<uint32_t>();
        w.xtmp = csr->lw_xtmp.as<int32_t>();
        w.tile = kLwTileMax; // about four tiles per wave slot of the chip, within the limits
        while (w.tile > kLwTileMin && D / w.tile < (int64_t)csr->num_cu * 128)
            w.tile >>= 1;
        w.tiles_bound = D / w.tile + c.k;
        BMS_TRY(csr->lw_tiles.ensure((size_t)w.tiles_bound * (sizeof(int64_t) + sizeof(uint32_t)) + 64));
        BMS_TRY(csr->lw_rowcnt.ensure((size_t)rows_bound * sizeof(uint32_t)));
        w.tile_row = csr->lw_tiles.as<int64_t>();
        w.tile_cnt = reinterpret_cast<uint32_t *>(w.tile_row + w.tiles_bound);
        w.first_cnt = csr->lw_rowcnt.as<uint32_t>();
        BMS_TRY(prof.begin("ldw_bounds", h));
        launch_ldw_bounds(c.launch, w);
        BMS_TRY(prof.end());
        BMS_TRY(prof.begin("ldw_accumulate", h));
        if (launch_ldw_accumulate(c.launch, w) != 0)
            return fail(BMS_EHIP, "launch of the LDS accumulation kernel was refused");
        launch_offsets_from_counts(c.launch, w.mb_count, c.k, w.p_off, slot(c, h, 2));
        BMS_TRY(prof.end());
        // nnz(P) sizes P and its prefix sums.  When its bound min(D, k n) is modest the buffers take the bound
        // and the size is read back with everything else at the end of the call; else it is read back now.
        int64_t pnnz = std::max<int64_t>(std::min<int64_t>(D, (int64_t)c.k * n1), 1);
        if (no_wait) {
            pnnz = std::min<int64_t>(pnnz, with_margin(c.res->hint_pnnz[h]));
        } else if (pnnz > kNoWaitEntries) {
            BMS_TRY(read_scalars(c));
            pnnz = host_slot(c, h, 2);
        }
        w.p_cap = pnnz;
        BMS_TRY(hb.p_col.ensure((size_t)std::max<int64_t>(pnnz, 1) * sizeof(int32_t)));
        BMS_TRY(hb.p_cnt.ensure((size_t)std::max<int64_t>(pnnz, 1) * sizeof(uint32_t)));
        BMS_TRY(csr->ld_prefix.ensure((size_t)std::max<int64_t>(pnnz, 1) * sizeof(uint64_t)));
        w.p_col = hb.p_col.as<int32_t>();
        w.p_cnt = hb.p_cnt.as<uint32_t>();
        w.prefix = csr->ld_prefix.as<uint64_t>();
        BMS_TRY(prof.begin("ldw_p_copy", h));
        launch_ldw_p_copy(c.launch, w);
        BMS_TRY(prof.end());
        // NORM (implicit) + SAMPLE
        BMS_TRY(prof.begin("ldw_draw", h));
        launch_ldw_draw(c.launch, w);
        launch_offsets_from_counts(c.launch, w.mb_count, c.k, w.mb_coloff, slot(c, h, 1));
        launch_ldw_sel_copy(c.launch, w);
        BMS_TRY(prof.end());
        // EXTRACT
        BMS_TRY(prof.begin("ldw_extract", h));
        launch_ldw_extract(c.launch, w);
        launch_scan_i64(c.launch, w.out_rowptr, mb_rowoff + c.k, slot(c, h, 0), nullptr, nullptr, rows_bound);
        BMS_TRY(prof.end());
        // nnz sizes the column buffer: same rule with the bound min(D, rows * s)
        int64_t nnz = std::min<int64_t>(D, rows_bound * std::min<int64_t>(s, n1));
        if (no_wait) {
            nnz = std::min<int64_t>(nnz, with_margin(c.res->hint_nnz[h]));
        } else if (nnz > kNoWaitEntries) {
            BMS_TRY(read_scalars(c));
            nnz = host_slot(c, h, 0);
        }
        w.col_cap = std::max<int64_t>(nnz, 1);
        BMS_TRY(hb.col.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(int32_t)));
        w.out_col = hb.col.as<int32_t>();
        BMS_TRY(prof.begin("ldw_extract_copy", h));
        launch_ldw_extract_copy(c.launch, w);
        BMS_TRY(prof.end());

        hb.view = bms_hop_view{}; // the sizes follow after the last read-back
        hb.view.mb_rowoff = mb_rowoff;
        hb.view.row_vertex = row_vertex;
        hb.view.rowptr = hb.rowptr.as<int64_t>();
        hb.view.col = hb.col.as<int32_t>();
        hb.view.mb_coloff = hb.mb_coloff.as<int64_t>();
        hb.view.col_vertex = hb.col_vertex.as<int32_t>();
        hb.view.p_off = hb.p_off.as<int64_t>();
        hb.view.p_col = hb.p_col.as<int32_t>();
        hb.view.p_cnt = hb.p_cnt.as<uint32_t>();

        row_vertex = hb.col_vertex.as<int32_t>();
        mb_rowoff = hb.mb_coloff.as<int64_t>();
        rows_bound = std::max<int64_t>(ncols_bound, 1);
    }
    BMS_TRY(read_scalars(c));
    if (no_wait) {
        BMS_TRY(seed_flag_error(c));
        if ((int32_t)(csr->host_pinned[60] & 0xFFFFFFFF)) { // a size went past what the remembered call needed
            *redo = true;
            return BMS_OK;
        }
    }
    c.res->hint_gathered.assign((size_t)c.L, 0);
    c.res->hint_pnnz.assign((size_t)c.L, 0);
    c.res->hint_nnz.assign((size_t)c.L, 0);
    for (int32_t h = 0; h < c.L; ++h) {
        bms_hop_view &v = c.res->hops[h].view;
        v.nnz = host_slot(c, h, 0);
        v.ncols = host_slot(c, h, 1);
        v.pnnz = host_slot(c, h, 2);
        v.rows = h == 0 ? (int64_t)c.k * c.b : c.res->hops[h - 1].view.ncols;
        c.res->hint_nnz[h] = v.nnz;
        c.res->hint_pnnz[h] = v.pnnz;
        c.res->hint_gathered[h] = host_slot(c, h, 3);
    }
    c.res->hint_csr = csr;
    c.res->hint_shape = shape;
    BMS_TRY(prof.finish());
    return BMS_OK;
}

int sample_ladies_windows_impl(CallCtx &c, const int32_t *batches, const int32_t *s_per_layer)
{
    bool redo = false;
    c.res->attempts = 1;
    BMS_TRY(sample_ladies_windows_once(c, batches, s_per_layer, true, &redo));
    if (!redo)
        return BMS_OK;
    c.res->stages.clear();
    c.res->events_used = 0;
    c.res->attempts = 2;
    BMS_TRY(sample_ladies_windows_once(c, batches, s_per_layer, false, &redo));
    return BMS_OK;
}

int sample_ladies_impl(CallCtx &c, const int32_t *batches, const int32_t *s_per_layer)
{
    if (ladies_windows_apply(c, s_per_layer))
        return sample_ladies_windows_impl(c, batches, s_per_layer);
    bms_csr *csr = c.csr;
    Profiler prof{c.res, c.stream, (c.flags & (BMS_PROFILE | BMS_PROFILE_MAIN)) != 0, (c.flags & BMS_PROFILE) == 0};
    BMS_TRY(setup_vset(c));

    // dense per-minibatch counters e_v, all zero between hops and between calls
    const size_t cbytes = (size_t)c.k * (size_t)std::max<int64_t>(csr->n, 1) * sizeof(uint32_t);
    const size_t vbytes = csr->vs_words.cap + csr->vs_prefix.cap + csr->vs_chunks.cap;
    if ((int64_t)(cbytes + vbytes) > c.scratch_limit)
        return fail(BMS_ENOMEM,
                    "dense counters for k=%d minibatches over n=%lld vertices need %zu bytes of scratch (plus %zu for "
                    "the vertex sets), limit is %lld: raise bms_opts.scratch_limit or sample fewer minibatches per call",
                    c.k, (long long)csr->n, cbytes, vbytes, (long long)c.scratch_limit);
    BMS_TRY(csr->ld_counters.ensure(cbytes));
    if (csr->ld_counters.grew)
        csr->ld_clean = false;
    if (!csr->ld_clean)
        HIP_TRY(hipMemsetAsync(csr->ld_counters.p, 0, csr->ld_counters.cap, c.stream));
    csr->ld_clean = false;
    const int32_t nchunk = (int32_t)((std::max<int64_t>(csr->n, 1) + kPChunk - 1) / kPChunk);
    BMS_TRY(csr->ld_chunks.ensure(((size_t)c.k * nchunk + c.k) * sizeof(int64_t)));
    BMS_TRY(csr->ld_ptileoff.ensure(((size_t)c.k + 1) * sizeof(int64_t)));

    BMS_TRY(stage_seeds(c, batches, prof));

    int64_t rows_bound = (int64_t)c.k * c.b;
    const int32_t *row_vertex = c.res->hops[0].row_vertex.as<int32_t>();
    const int64_t *mb_rowoff = c.res->hops[0].mb_rowoff.as<int64_t>();

    for (int32_t h = 0; h < c.L; ++h) {
        HopBufs &hb = c.res->hops[h];
        const int32_t s = s_per_layer[h];
        const int64_t ncols_bound = (int64_t)c.k * std::min<int64_t>(s, std::max<int64_t>(csr->n, 1));
        BMS_TRY(csr->row_beg.ensure((size_t)rows_bound * sizeof(int64_t)));
        BMS_TRY(csr->ld_gather_off.ensure((size_t)(rows_bound + 1) * sizeof(int64_t)));
        BMS_TRY(csr->ld_row_mb.ensure((size_t)rows_bound * sizeof(int32_t)));
        BMS_TRY(hb.rowptr.ensure((size_t)(rows_bound + 1) * sizeof(int64_t)));
        BMS_TRY(hb.mb_coloff.ensure(((size_t)c.k + 1) * sizeof(int64_t)));
        BMS_TRY(hb.col_vertex.ensure((size_t)ncols_bound * sizeof(int32_t)));
        BMS_TRY(hb.p_off.ensure(((size_t)c.k + 1) * sizeof(int64_t)));

        LdHop a{};
        a.A_rowptr = csr->rowptr;
        a.A_col = csr->col;
        a.n = csr->n;
        a.k = c.k;
        a.s = s;
        a.squared = (c.flags & BMS_LADIES_SQUARED) ? 1 : 0;
        a.hopkey = hop_key(c.seed, h);
        a.mb_base = c.mb_base;
        a.row_vertex = row_vertex;
        a.mb_rowoff = mb_rowoff;
        a.rows_bound = rows_bound;
        a.row_beg = csr->row_beg.as<int64_t>();
        a.gather_off = csr->ld_gather_off.as<int64_t>();
        a.row_mb = csr->ld_row_mb.as<int32_t>();
        a.gather_tiles = csr->scalars.as<int64_t>() + 62;
        a.counters = csr->ld_counters.as<uint32_t>();
        a.p_chunks = csr->ld_chunks.as<int64_t>();
        a.nchunk = nchunk;
        a.p_off = hb.p_off.as<int64_t>();
        a.p_tileoff = csr->ld_ptileoff.as<int64_t>();
        a.out_rowptr = hb.rowptr.as<int64_t>();

        // P = Q A
        BMS_TRY(prof.begin("ld_rows", h));
        launch_ld_rows(c.launch, a, slot(c, h, 3));
        BMS_TRY(prof.end());
        BMS_TRY(read_scalars(c)); // D sizes the tile arrays of the gathered order
        if (h == 0)
            BMS_TRY(seed_flag_error(c));
        const int64_t D = host_slot(c, h, 3);
        BMS_TRY(csr->tile_off.ensure((size_t)(D / kGatherTile + 3) * sizeof(int64_t)));
        a.tile_off = csr->tile_off.as<int64_t>();
        BMS_TRY(prof.begin("ld_accumulate", h));
        launch_ld_accumulate(c.launch, a);
        BMS_TRY(prof.end());
        BMS_TRY(prof.begin("ld_p_count", h));
        launch_ld_p_count(c.launch, a, slot(c, h, 2));
        BMS_TRY(prof.end());
        BMS_TRY(read_scalars(c)); // pnnz sizes P and its prefix sums
        const int64_t pnnz = host_slot(c, h, 2);
        BMS_TRY(hb.p_col.ensure((size_t)std::max<int64_t>(pnnz, 1) * sizeof(int32_t)));
        BMS_TRY(hb.p_cnt.ensure((size_t)std::max<int64_t>(pnnz, 1) * sizeof(uint32_t)));
        BMS_TRY(csr->ld_prefix.ensure((size_t)std::max<int64_t>(pnnz, 1) * sizeof(uint64_t)));
        BMS_TRY(csr->ld_tilesum.ensure((size_t)(pnnz / kPTile + c.k + 1) * sizeof(uint64_t)));
        a.p_col = hb.p_col.as<int32_t>();
        a.p_cnt = hb.p_cnt.as<uint32_t>();
        a.prefix = csr->ld_prefix.as<uint64_t>();
        a.p_tilesum = csr->ld_tilesum.as<uint64_t>();
        a.pnnz_bound = pnnz;
        BMS_TRY(prof.begin("ld_p_fill", h));
        launch_ld_p_fill(c.launch, a);
        BMS_TRY(prof.end());
        // NORM (implicit) + SAMPLE
        BMS_TRY(prof.begin("ld_prefix", h));
        launch_ld_prefix(c.launch, a);
        BMS_TRY(prof.end());
        BMS_TRY(prof.begin("ld_draw", h));
        launch_ld_draw(c.launch, a, c.vs);
        BMS_TRY(prof.end());
        BMS_TRY(prof.begin("vset_rank", h));
        launch_vset_rank(c.launch, c.vs, c.k, hb.mb_coloff.as<int64_t>(), hb.col_vertex.as<int32_t>(), slot(c, h, 1));
        BMS_TRY(prof.end());
        BMS_TRY(prof.begin("ld_clear", h));
        launch_ld_clear_counters(c.launch, a);
        BMS_TRY(prof.end());
        // EXTRACT
        BMS_TRY(prof.begin("ld_extract_count", h));
        launch_ld_extract_count(c.launch, a, c.vs, slot(c, h, 0));
        BMS_TRY(prof.end());
        BMS_TRY(read_scalars(c)); // nnz sizes the column buffer
        const int64_t nnz = host_slot(c, h, 0);
        BMS_TRY(hb.col.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(int32_t)));
        a.out_col = hb.col.as<int32_t>();
        BMS_TRY(prof.begin("ld_extract_fill", h));
        launch_ld_extract_fill(c.launch, a, c.vs);
        BMS_TRY(prof.end());
        BMS_TRY(prof.begin("vset_clear", h));
        launch_vset_clear(c.launch, c.vs, c.k, hb.mb_coloff.as<int64_t>(), hb.col_vertex.as<int32_t>(), ncols_bound);
        BMS_TRY(prof.end());

        hb.view = bms_hop_view{};
        hb.view.nnz = nnz;
        hb.view.pnnz = pnnz;
        hb.view.ncols = host_slot(c, h, 1); // written before the last read-back of this hop
        hb.view.mb_rowoff = mb_rowoff;
        hb.view.row_vertex = row_vertex;
        hb.view.rowptr = hb.rowptr.as<int64_t>();
        hb.view.col = hb.col.as<int32_t>();
        hb.view.mb_coloff = hb.mb_coloff.as<int64_t>();
        hb.view.col_vertex = hb.col_vertex.as<int32_t>();
        hb.view.p_off = hb.p_off.as<int64_t>();
        hb.view.p_col = hb.p_col.as<int32_t>();
        hb.view.p_cnt = hb.p_cnt.as<uint32_t>();
        hb.view.rows = h == 0 ? (int64_t)c.k * c.b : c.res->hops[h - 1].view.ncols;

        row_vertex = hb.col_vertex.as<int32_t>();
        mb_rowoff = hb.mb_coloff.as<int64_t>();
        rows_bound = std::max<int64_t>(ncols_bound, 1);
    }
    HIP_TRY(hipStreamSynchronize(c.stream));
    BMS_TRY(prof.finish());
    csr->vs_clean = true;
    csr->ld_clean = true;
    return BMS_OK;
}

} // namespace

extern "C" {

int bms_csr_load(const int64_t *rowptr, const int32_t *col, int64_t n, int64_t nnz, int location, bms_csr **out)
{
    if (!rowptr || !out || (!col && nnz > 0))
        return fail(BMS_EINVAL, "null argument");
    if (n < 0 || nnz < 0 || n > 0x7FFFFFFFLL)
        return fail(BMS_EINVAL, "n=%lld nnz=%lld out of range (vertex ids are int32)", (long long)n, (long long)nnz);
    if (location != BMS_HOST && location != BMS_DEVICE_BORROW && location != BMS_DEVICE_COPY)
        return fail(BMS_EINVAL, "unknown location %d", location);
    bms_csr *c = new (std::nothrow) bms_csr();
    if (!c)
        return fail(BMS_ENOMEM, "host allocation failed");
    auto bail = [&](int rc) {
        bms_free(c);
        return rc;
    };
    hipError_t e = hipGetDevice(&c->device);
    if (e != hipSuccess)
        return bail(fail(BMS_EHIP, "hipGetDevice failed: %s", hipGetErrorString(e)));
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, c->device) == hipSuccess && prop.multiProcessorCount > 0)
        c->num_cu = prop.multiProcessorCount;
    {   // set-up of the device's static scratch (used by bms_result_minibatch_offsets); a failure is reported there
        int64_t *unused = nullptr;
        (void)scratch_address(c->device, &unused);
    }
    c->n = n;
    c->nnz = nnz;
    if (location == BMS_DEVICE_BORROW) {
        c->rowptr = rowptr;
        c->col = col;
    } else {
        const hipMemcpyKind kind = location == BMS_HOST ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice;
        int rc = c->own_rowptr.ensure((size_t)(n + 1) * sizeof(int64_t));
        if (rc == BMS_OK)
            rc = c->own_col.ensure((size_t)std::max<int64_t>(nnz, 1) * sizeof(int32_t));
        if (rc != BMS_OK)
            return bail(rc);
        e = hipMemcpy(c->own_rowptr.p, rowptr, (size_t)(n + 1) * sizeof(int64_t), kind);
        if (e == hipSuccess && nnz > 0)
            e = hipMemcpy(c->own_col.p, col, (size_t)nnz * sizeof(int32_t), kind);
        if (e != hipSuccess)
            return bail(fail(BMS_EHIP, "copying the CSR arrays failed: %s", hipGetErrorString(e)));
        c->rowptr = c->own_rowptr.as<int64_t>();
        c->col = c->own_col.as<int32_t>();
    }
    // structure check on the device
    int rc = c->scalars.ensure(64 * sizeof(int64_t));
    if (rc != BMS_OK)
        return bail(rc);
    e = hipMemset(c->scalars.p, 0, 64 * sizeof(int64_t));
    if (e != hipSuccess)
        return bail(fail(BMS_EHIP, "hipMemset failed: %s", hipGetErrorString(e)));
    Launch L{nullptr, c->num_cu};
    int32_t *flag = reinterpret_cast<int32_t *>(c->scalars.as<int64_t>() + 1);
    launch_csr_check(L, c->rowptr, c->col, n, nnz, flag, reinterpret_cast<unsigned long long *>(c->scalars.p));
    int64_t host[2] = {0, 0};
    e = hipMemcpy(host, c->scalars.p, sizeof(host), hipMemcpyDeviceToHost);
    if (e != hipSuccess)
        return bail(fail(BMS_EHIP, "CSR verification failed to run: %s", hipGetErrorString(e)));
    const int32_t bad = (int32_t)(host[1] & 0xFFFFFFFF);
    if (bad & 1)
        return bail(fail(BMS_EFORMAT, "rowptr is not a monotone sequence from 0 to nnz"));
    if (bad & 2)
        return bail(fail(BMS_EFORMAT, "a column index lies outside [0, n)"));
    if (bad & 4)
        return bail(fail(BMS_EFORMAT, "a row is not strictly ascending (unsorted or duplicate column)"));
    c->max_degree = host[0];
    *out = c;
    return BMS_OK;
}

int bms_csr_info(const bms_csr *csr, int64_t *n, int64_t *nnz, int64_t *max_degree)
{
    if (!csr || csr->tag != kTagCsr)
        return fail(BMS_EINVAL, "not a csr handle");
    if (n)
        *n = csr->n;
    if (nnz)
        *nnz = csr->nnz;
    if (max_degree)
        *max_degree = csr->max_degree;
    return BMS_OK;
}

int bms_csr_held_bytes(const bms_csr *csr, int64_t *bytes)
{
    if (!csr || csr->tag != kTagCsr || !bytes)
        return fail(BMS_EINVAL, "not a csr handle, or no place for the answer");
    size_t sum = 0;
    for (const DevBuf *b : csr->bufs)
        sum += b->p ? b->cap : 0;
    *bytes = (int64_t)sum;
    return BMS_OK;
}

int bms_sample_nodewise(bms_csr *csr, const int32_t *batches, int32_t k, int32_t b, const int32_t *fanouts, int32_t L,
                        uint64_t seed, const bms_opts *opts, bms_result **out)
{
    BMS_TRY(check_common(csr, batches, k, b, fanouts, L, opts, out));
    if (L > kMaxHops)
        return fail(BMS_EINVAL, "at most %d hops are supported", kMaxHops);
    for (int32_t h = 0; h < L; ++h)
        if (fanouts[h] > kMaxSampledFanout && (int64_t)fanouts[h] < csr->max_degree)
            return fail(BMS_EINVAL,
                        "fanout %d at hop %d: a fanout above %d must be >= the largest degree (%lld) so that no row "
                        "needs sampling",
                        fanouts[h], h, kMaxSampledFanout, (long long)csr->max_degree);
    if (opts && (opts->flags & BMS_NODEWISE_REPLACE))
        for (int32_t h = 0; h < L; ++h)
            if (fanouts[h] > kMaxSampledFanout)
                return fail(BMS_EINVAL, "fanout %d at hop %d: with BMS_NODEWISE_REPLACE a fanout is at most %d",
                            fanouts[h], h, kMaxSampledFanout);
    CallCtx c{};
    int rc = begin_call(c, csr, k, b, L, seed, opts);
    if (rc == BMS_OK)
        rc = sample_nodewise_impl(c, batches, fanouts);
    if (rc != BMS_OK)
        return abort_call(c, rc);
    *out = c.res;
    return BMS_OK;
}

int bms_sample_ladies(bms_csr *csr, const int32_t *batches, int32_t k, int32_t b, const int32_t *s_per_layer,
                      int32_t L, uint64_t seed, const bms_opts *opts, bms_result **out)
{
    BMS_TRY(check_common(csr, batches, k, b, s_per_layer, L, opts, out));
    if (L > kMaxHops)
        return fail(BMS_EINVAL, "at most %d hops are supported", kMaxHops);
    if (opts && (opts->flags & (BMS_UNION_DST | BMS_NODEWISE_REPLACE)))
        return fail(BMS_EINVAL, "BMS_UNION_DST and BMS_NODEWISE_REPLACE apply to node-wise sampling only");
    CallCtx c{};
    int rc = begin_call(c, csr, k, b, L, seed, opts);
    if (rc == BMS_OK)
        rc = sample_ladies_impl(c, batches, s_per_layer);
    if (rc != BMS_OK)
        return abort_call(c, rc);
    *out = c.res;
    return BMS_OK;
}

int bms_result_wait(bms_result *res)
{
    if (!res || res->tag != kTagResult)
        return fail(BMS_EINVAL, "not a result handle");
    return settle_result(res);
}

int bms_result_ready(const bms_result *res)
{
    if (!res || res->tag != kTagResult)
        return fail(BMS_EINVAL, "not a result handle");
    if (!res->pending)
        return 1;
    const hipError_t e = hipEventQuery(res->done_ev);
    if (e == hipErrorNotReady) {
        (void)hipGetLastError();
        return 0;
    }
    return 1;
}

int bms_result_attempts(const bms_result *res, int32_t *attempts)
{
    if (!res || res->tag != kTagResult || !attempts)
        return fail(BMS_EINVAL, "not a result handle, or no place for the answer");
    BMS_TRY(settle_result(const_cast<bms_result *>(res)));
    *attempts = res->attempts;
    return BMS_OK;
}

int bms_result_info(const bms_result *res, int32_t *k, int32_t *L)
{
    if (!res || res->tag != kTagResult)
        return fail(BMS_EINVAL, "not a result handle");
    BMS_TRY(settle_result(const_cast<bms_result *>(res)));
    if (k)
        *k = res->k;
    if (L)
        *L = res->L;
    return BMS_OK;
}

int bms_result_hop(const bms_result *res, int32_t hop, bms_hop_view *view)
{
    if (!res || res->tag != kTagResult || !view)
        return fail(BMS_EINVAL, "not a result handle, or null view");
    BMS_TRY(settle_result(const_cast<bms_result *>(res)));
    if (hop < 0 || hop >= res->L)
        return fail(BMS_EINVAL, "hop %d outside [0, %d)", hop, res->L);
    *view = res->hops[hop].view;
    return BMS_OK;
}

int bms_result_minibatch(bms_result *res, int32_t hop, int32_t i, bms_mb_view *view)
{
    if (!res || res->tag != kTagResult || !view)
        return fail(BMS_EINVAL, "not a result handle, or null view");
    BMS_TRY(settle_result(res));
    if (hop < 0 || hop >= res->L)
        return fail(BMS_EINVAL, "hop %d outside [0, %d)", hop, res->L);
    if (i < 0 || i >= res->k)
        return fail(BMS_EINVAL, "minibatch %d outside [0, %d)", i, res->k);
    const size_t stride = (size_t)res->k + 1;
    if (res->mb_offsets.empty()) {
        HIP_TRY(hipSetDevice(res->device));
        std::vector<int64_t> host((size_t)res->L * 3 * stride);
        BMS_TRY(res->mb_edge_tmp.ensure(stride * sizeof(int64_t)));
        for (int32_t h = 0; h < res->L; ++h) {
            const bms_hop_view &v = res->hops[h].view;
            int64_t *dst = host.data() + (size_t)h * 3 * stride;
            launch_mb_edge_offsets(nullptr, v.rowptr, v.mb_rowoff, res->k, res->mb_edge_tmp.as<int64_t>());
            HIP_TRY(hipMemcpy(dst, v.mb_rowoff, stride * sizeof(int64_t), hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(dst + stride, res->mb_edge_tmp.p, stride * sizeof(int64_t), hipMemcpyDeviceToHost));
            HIP_TRY(hipMemcpy(dst + 2 * stride, v.mb_coloff, stride * sizeof(int64_t), hipMemcpyDeviceToHost));
        }
        res->mb_offsets.swap(host);
    }
    const bms_hop_view &v = res->hops[hop].view;
    const int64_t *off = res->mb_offsets.data() + (size_t)hop * 3 * stride;
    bms_mb_view m{};
    m.row0 = off[i];
    m.rows = off[i + 1] - off[i];
    m.edge0 = off[stride + i];
    m.nnz = off[stride + i + 1] - off[stride + i];
    m.col0 = off[2 * stride + i];
    m.ncols = off[2 * stride + i + 1] - off[2 * stride + i];
    m.row_vertex = v.row_vertex + m.row0;
    m.rowptr = v.rowptr + m.row0;
    m.col = v.col + m.edge0;
    m.col_vertex = v.col_vertex + m.col0;
    m.row_self = v.row_self ? v.row_self + m.row0 : nullptr;
    *view = m;
    return BMS_OK;
}

int bms_result_minibatch_offsets(const bms_result *res, int32_t hop, int64_t *row_off, int64_t *edge_off,
                                 int64_t *col_off, void *stream)
{
    if (!res || res->tag != kTagResult || !row_off || !edge_off || !col_off)
        return fail(BMS_EINVAL, "not a result handle, or null output array");
    BMS_TRY(settle_result(const_cast<bms_result *>(res)));
    if (hop < 0 || hop >= res->L)
        return fail(BMS_EINVAL, "hop %d outside [0, %d)", hop, res->L);
    if (res->k > kNoAllocMaxK)
        return fail(BMS_EINVAL, "k=%d minibatches: this entry point holds at most %d (its scratch is a fixed array); "
                                "use bms_result_minibatch", res->k, kNoAllocMaxK);
    int device = 0;
    HIP_TRY(hipGetDevice(&device));
    if (device != res->device)
        return fail(BMS_EINVAL, "the result lives on device %d, the current device is %d", res->device, device);
    int64_t *tmp = nullptr;
    BMS_TRY(scratch_address(device, &tmp));
    const bms_hop_view &v = res->hops[hop].view;
    const size_t bytes = ((size_t)res->k + 1) * sizeof(int64_t);
    hipStream_t st = (hipStream_t)stream;
    launch_mb_edge_offsets(st, v.rowptr, v.mb_rowoff, res->k, tmp); // writes all k+1 values: nothing to clear
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipMemcpyAsync(edge_off, tmp, bytes, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(row_off, v.mb_rowoff, bytes, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(col_off, v.mb_coloff, bytes, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return BMS_OK;
}

int bms_result_stage(const bms_result *res, int32_t idx, const char **name, int32_t *hop, float *ms)
{
    if (!res || res->tag != kTagResult)
        return fail(BMS_EINVAL, "not a result handle");
    BMS_TRY(settle_result(const_cast<bms_result *>(res)));
    if (idx < 0 || idx >= (int32_t)res->stages.size())
        return BMS_EINVAL; // past the end: not an error worth a message
    const StageTime &st = res->stages[idx];
    if (name)
        *name = st.name;
    if (hop)
        *hop = st.hop;
    if (ms)
        *ms = st.ms;
    return BMS_OK;
}

void bms_free(void *handle)
{
    if (!handle)
        return;
    const uint32_t tag = *static_cast<const uint32_t *>(handle);
    if (tag == kTagCsr) {
        bms_csr *c = static_cast<bms_csr *>(handle);
        (void)hipSetDevice(c->device);
        for (DevBuf *b : c->bufs)
            b->release();
        if (c->host_pinned)
            (void)hipHostFree(c->host_pinned);
        c->tag = 0;
        delete c;
    } else if (tag == kTagResult) {
        bms_result *r = static_cast<bms_result *>(handle);
        result_release(r);
        r->tag = 0;
        delete r;
    }
}

int bms_fetch_features(const float *H, int64_t n, int32_t f, const int32_t *ids, int64_t m, float *out, void *stream)
{
    if (n < 0 || f < 1 || m < 0)
        return fail(BMS_EINVAL, "n=%lld f=%d m=%lld out of range", (long long)n, f, (long long)m);
    if (m == 0)
        return BMS_OK; // nothing to fetch: the pointers are not looked at
    if (!H || !out || !ids)
        return fail(BMS_EINVAL, "null argument");
    int device = 0;
    HIP_TRY(hipGetDevice(&device));
    // error flags in host memory that the kernel can write (nothing to allocate per call): a ring of kFlagSlots
    // words per device, one slot per call, so that fetches running at the same time on different streams do not
    // share a flag (a slot is reused after kFlagSlots further calls on the device)
    constexpr int kFlagSlots = 64;
    static int32_t *flags[64] = {nullptr};
    static uint32_t next_slot[64] = {0};
    static std::mutex flags_lock;
    int32_t *flag = nullptr;
    {
        std::lock_guard<std::mutex> guard(flags_lock);
        if (device < 0 || device >= 64)
            return fail(BMS_EINVAL, "device ordinal %d not supported", device);
        if (!flags[device])
            HIP_TRY(hipHostMalloc((void **)&flags[device], kFlagSlots * sizeof(int32_t), hipHostMallocMapped));
        flag = flags[device] + (next_slot[device]++ % kFlagSlots);
    }
    int32_t *flag_dev = nullptr;
    HIP_TRY(hipHostGetDevicePointer((void **)&flag_dev, flag, 0));
    hipDeviceProp_t prop;
    int num_cu = 256;
    static int cached_cu[64] = {0};
    if (!cached_cu[device] && hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount > 0)
        cached_cu[device] = prop.multiProcessorCount;
    if (cached_cu[device])
        num_cu = cached_cu[device];
    *flag = 0;
    launch_feature_fetch(Launch{(hipStream_t)stream, num_cu}, H, n, f, ids, m, out, flag_dev);
    HIP_TRY(hipGetLastError());
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    if (*flag)
        return fail(BMS_ERANGE, "a vertex id lies outside [0, %lld)", (long long)n);
    return BMS_OK;
}

int bms_aggregate_hop(const bms_result *res, int32_t hop, const float *X, int32_t f, int mean, float *out, void *stream)
{
    if (!res || res->tag != kTagResult)
        return fail(BMS_EINVAL, "not a result handle");
    BMS_TRY(settle_result(const_cast<bms_result *>(res)));
    if (hop < 0 || hop >= res->L)
        return fail(BMS_EINVAL, "hop %d outside [0, %d)", hop, res->L);
    if (f < 1)
        return fail(BMS_EINVAL, "f=%d must be >= 1", f);
    const bms_hop_view &v = res->hops[hop].view;
    if (v.rows == 0)
        return BMS_OK;
    if (!out || (!X && v.nnz > 0))
        return fail(BMS_EINVAL, "null argument");
    AggArgs a{};
    a.rows = v.rows;
    a.k = res->k;
    a.f = f;
    a.mean = mean;
    a.mb_rowoff = v.mb_rowoff;
    a.rowptr = v.rowptr;
    a.col = v.col;
    a.mb_coloff = v.mb_coloff;
    a.X = X;
    a.out = out;
    int device = 0, num_cu = 256;
    HIP_TRY(hipGetDevice(&device));
    HIP_TRY(hipDeviceGetAttribute(&num_cu, hipDeviceAttributeMultiprocessorCount, device));
    launch_aggregate(Launch{(hipStream_t)stream, num_cu > 0 ? num_cu : 256}, a);
    HIP_TRY(hipGetLastError());
    return BMS_OK;
}

const char *bms_strerror(int code)
{
    switch (code) {
    case BMS_OK: return "success";
    case BMS_EINVAL: return "invalid argument";
    case BMS_ERANGE: return "vertex id out of range, or seed repeated inside a minibatch";
    case BMS_EFORMAT: return "malformed CSR matrix";
    case BMS_ENOMEM: return "out of memory or scratch limit too small";
    case BMS_EHIP: return "HIP runtime error";
    case BMS_EAGAIN: return "the asynchronous call gave up on its kernel path: repeat the call";
    default: return "unknown error code";
    }
}

const char *bms_last_error(void) { return g_err; }

} // extern "C"
