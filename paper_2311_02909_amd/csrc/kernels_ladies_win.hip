// Layer-wise (LADIES) bulk sampling, Sec. 4.2 of arxiv 2311.02909: the path that accumulates the
// column counts of P = Q A in LDS.
//
// The rows of A are sorted by column, so the neighbours of a frontier row that fall into a window
// of 2^16 vertex ids form one contiguous piece of its adjacency list.  One hop, all k minibatches:
//   ldw_bounds      one wave per frontier row streams the row once and records where it crosses
//                   every window boundary (lower bounds, kept window-major so that the next
//                   kernel reads them coalesced)
//   ldw_accumulate  one workgroup per (minibatch, window): 2^16 packed 16-bit counters in LDS
//                   (128 KB); every row's piece of the window adds 1 per neighbour (e_v cannot
//                   exceed the number of frontier rows, which this path keeps below 2^16); the
//                   nonzero counters leave in ascending column order as (column, e_v) through a
//                   device-wide cursor
//   ldw_win_scan    per minibatch: columns and weight before every window
//   ldw_p_copy      windows copied to their place in P; inclusive prefix sums of the integer
//                   weights (e_v or e_v^2) on the way (NORM stays implicit: draws are integers
//                   below the row sum)
//   ldw_draw        SAMPLE (Sec. 4.2.2): one workgroup per minibatch: s draws, each the smallest t
//                   with prefix[t] > r, sorted in LDS, duplicates dropped -> sampled columns
//   ldw_extract     EXTRACT (Sec. 4.2.3): the sampled columns of the minibatch sit in an LDS hash
//                   table (column -> local index); one wave per frontier row streams the row a
//                   second time and keeps the neighbours found in the table ((Q_R A) Q_C), in
//                   row order; rows are then sized by a scan and copied to their place
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

constexpr int kWinIds = 1 << kWinShift;
constexpr int kWinWords = kWinIds / 2; // two 16-bit counters per LDS word
constexpr int kAccThreads = 1024;
constexpr int kAccWaves = kAccThreads / kWave;
constexpr int kWaveWords = kWinWords / kAccWaves; // counter words compacted by one wave
constexpr uint32_t kEmptySlot = 0xFFFFFFFFu;
constexpr int kHashSlots = 2 * kMaxWinSampled;    // load factor <= 1/2

__device__ inline uint64_t ldw_weight(uint32_t cnt, int squared)
{
    return squared ? (uint64_t)cnt * (uint64_t)cnt : (uint64_t)cnt;
}

// ---------------------------------------------------------------------------------------------
// bounds[w * rows_bound + r] = number of neighbours of row r with id < w * 2^16, w = 0..nwin
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ldw_bounds_kernel(LwHop a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t R = a.mb_rowoff[a.k];
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t r = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave; r < R; r += nwaves) {
        const uint32_t deg = (uint32_t)(a.gather_off[r + 1] - a.gather_off[r]);
        const int32_t *__restrict__ src = a.A_col + a.row_beg[r];
        uint32_t *__restrict__ out = a.bounds + r;
        // position deg acts as one more entry that lies in window nwin: it closes every window left
        int32_t carry = -1; // window of the entry before the ones in flight
        for (uint32_t j0 = 0; j0 <= deg; j0 += 4 * kWave) {
            int32_t wv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t j = j0 + u * kWave + lane;
                wv[u] = j < deg ? (src[j] >> kWinShift) : a.nwin;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t j = j0 + u * kWave + lane;
                int32_t pw = __shfl_up(wv[u], 1, kWave);
                if (lane == 0)
                    pw = carry;
                if (j <= deg)
                    for (int32_t w = pw + 1; w <= wv[u]; ++w)
                        out[(int64_t)w * a.rows_bound] = j;
                carry = __shfl(wv[u], kWave - 1, kWave);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// P = Q A for one (minibatch, window) per workgroup
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kAccThreads) void ldw_accumulate_kernel(LwHop a)
{
    extern __shared__ uint32_t lds[];
    uint32_t *cnt = lds;                                               // kWinWords packed counters
    uint64_t *wave_wt = reinterpret_cast<uint64_t *>(lds + kWinWords); // kAccWaves
    uint32_t *wave_nz = lds + kWinWords + 2 * kAccWaves;               // kAccWaves
    uint64_t *base_s = reinterpret_cast<uint64_t *>(lds + kWinWords + 3 * kAccWaves); // 1
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t nblk = (int64_t)a.k * a.nwin;
    for (int64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const int i = (int)(blk / a.nwin), w = (int)(blk % a.nwin);
        const int64_t r0 = a.mb_rowoff[i], r1 = a.mb_rowoff[i + 1];
        for (int x = tid; x < kWinWords; x += kAccThreads)
            cnt[x] = 0;
        __syncthreads();
        const uint32_t *__restrict__ lo_b = a.bounds + (int64_t)w * a.rows_bound;
        const uint32_t *__restrict__ hi_b = lo_b + a.rows_bound;
        const int32_t id0 = w << kWinShift;
        const int sub = lane & 15, gbase = lane & 48;
        for (int64_t base = r0 + (int64_t)wave * kWave; base < r1; base += (int64_t)kAccWaves * kWave) {
            const int64_t r = base + lane;
            uint32_t len = 0;
            int64_t addr = 0;
            if (r < r1) {
                const uint32_t b0 = lo_b[r];
                len = hi_b[r] - b0;
                addr = a.row_beg[r] + b0;
            }
            if (__ballot(len != 0) == 0)
                continue;
            // four groups of 16 lanes; group g walks the pieces held by lanes 16 g .. 16 g + 15
#pragma unroll 4
            for (int t = 0; t < 16; ++t) {
                const uint32_t l = __shfl(len, gbase + t, kWave);
                const int64_t ad = __shfl(addr, gbase + t, kWave);
                for (uint32_t e = sub; e < l; e += 16) {
                    const uint32_t v = (uint32_t)(a.A_col[ad + e] - id0);
                    atomicAdd(&cnt[v >> 1], 1u << ((v & 1u) * 16));
                }
            }
        }
        __syncthreads();
        // each wave compacts kWaveWords consecutive words: first how many, then where, then the entries
        const uint32_t *__restrict__ mine = cnt + wave * kWaveWords;
        uint32_t nz = 0;
        uint64_t wt = 0;
        for (int it = 0; it < kWaveWords / kWave; ++it) {
            const uint32_t x = mine[it * kWave + lane];
            const uint32_t lo = x & 0xFFFFu, hi = x >> 16;
            nz += (lo != 0) + (hi != 0);
            wt += ldw_weight(lo, a.squared) + ldw_weight(hi, a.squared);
        }
        nz = wave_sum(nz);
        wt = wave_sum(wt);
        if (lane == 0) {
            wave_nz[wave] = nz;
            wave_wt[wave] = wt;
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t total = 0;
            uint64_t wsum = 0;
            for (int x = 0; x < kAccWaves; ++x) {
                const uint32_t c = wave_nz[x];
                wave_nz[x] = total; // exclusive
                total += c;
                wsum += wave_wt[x];
            }
            const uint64_t base = total ? atomicAdd(a.cursor, (unsigned long long)total) : 0ull;
            *base_s = base;
            a.win_cnt[blk] = total;
            a.win_wt[blk] = wsum;
            a.win_base[blk] = (int64_t)base;
        }
        __syncthreads();
        if (nz) { // uniform per wave
            int64_t run = (int64_t)*base_s + wave_nz[wave];
            const uint64_t below = (1ull << lane) - 1ull;
            for (int it = 0; it < kWaveWords / kWave; ++it) {
                const int word = wave * kWaveWords + it * kWave + lane;
                const uint32_t x = cnt[word];
                const uint32_t lo = x & 0xFFFFu, hi = x >> 16;
                const uint64_t mlo = __ballot(lo != 0), mhi = __ballot(hi != 0);
                if ((mlo | mhi) == 0)
                    continue;
                int64_t pos = run + __popcll(mlo & below) + __popcll(mhi & below);
                if (lo) {
                    a.tmp_col[pos] = id0 + 2 * word;
                    a.tmp_cnt[pos] = lo;
                    ++pos;
                }
                if (hi) {
                    a.tmp_col[pos] = id0 + 2 * word + 1;
                    a.tmp_cnt[pos] = hi;
                }
                run += __popcll(mlo) + __popcll(mhi);
            }
        }
        __syncthreads();
    }
}

// one workgroup per minibatch: columns and weight before each window; columns of the minibatch
__global__ __launch_bounds__(256) void ldw_win_scan_kernel(LwHop a)
{
    __shared__ uint64_t smem[4];
    __shared__ uint64_t carry_c, carry_w;
    const int i = blockIdx.x, tid = threadIdx.x;
    if (tid == 0) {
        carry_c = 0;
        carry_w = 0;
    }
    __syncthreads();
    for (int base = 0; base < a.nwin; base += 256) {
        const int w = base + tid;
        const int64_t x = (int64_t)i * a.nwin + w;
        const uint64_t c = w < a.nwin ? a.win_cnt[x] : 0u;
        const uint64_t wt = w < a.nwin ? a.win_wt[x] : 0u;
        uint64_t tc, tw;
        const uint64_t ec = block_exclusive_scan<uint64_t, 256>(c, smem, tc);
        const uint64_t ew = block_exclusive_scan<uint64_t, 256>(wt, smem, tw);
        const uint64_t cc = carry_c, cw = carry_w;
        if (w < a.nwin) {
            a.win_poff[x] = (int64_t)(cc + ec);
            a.win_woff[x] = cw + ew;
        }
        __syncthreads();
        if (tid == 0) {
            carry_c = cc + tc;
            carry_w = cw + tw;
        }
        __syncthreads();
    }
    if (tid == 0)
        a.mb_count[i] = (int64_t)carry_c;
}

// windows to their place in P, with the inclusive prefix sums of the weights
__global__ __launch_bounds__(256) void ldw_p_copy_kernel(LwHop a)
{
    __shared__ uint64_t smem[4];
    const int tid = threadIdx.x;
    const int64_t nblk = (int64_t)a.k * a.nwin;
    for (int64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const uint32_t cw = a.win_cnt[blk];
        if (cw == 0)
            continue;
        const int i = (int)(blk / a.nwin);
        const int64_t src = a.win_base[blk];
        const int64_t dst = a.p_off[i] + a.win_poff[blk];
        uint64_t carry = a.win_woff[blk];
        for (uint32_t x0 = 0; x0 < cw; x0 += 1024) {
            uint32_t c[4];
            int32_t col[4];
            uint64_t mine = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t x = x0 + tid * 4 + q;
                c[q] = 0;
                col[q] = 0;
                if (x < cw) {
                    c[q] = a.tmp_cnt[src + x];
                    col[q] = a.tmp_col[src + x];
                }
                mine += ldw_weight(c[q], a.squared);
            }
            uint64_t total;
            uint64_t run = carry + block_exclusive_scan<uint64_t, 256>(mine, smem, total);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t x = x0 + tid * 4 + q;
                run += ldw_weight(c[q], a.squared);
                if (x < cw) {
                    a.p_col[dst + x] = col[q];
                    a.p_cnt[dst + x] = c[q];
                    a.prefix[dst + x] = run;
                }
            }
            carry += total;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// SAMPLE: one workgroup per minibatch
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void ldw_draw_kernel(LwHop a)
{
    __shared__ uint32_t key[kMaxWinSampled];
    __shared__ uint32_t smem[16];
    const int i = blockIdx.x, tid = threadIdx.x;
    const int64_t p0 = a.p_off[i], C = a.p_off[i + 1] - p0;
    uint32_t M = 1024; // sorted size: a power of two >= s, at least one slot per thread
    while (M < (uint32_t)a.s)
        M <<= 1;
    const uint64_t *__restrict__ pre = a.prefix + p0;
    const uint64_t W = C > 0 ? pre[C - 1] : 0;
    const uint64_t rk = row_key(a.hopkey, a.mb_base + (uint32_t)i, kNoVertex);
    for (uint32_t j = tid; j < M; j += 1024) {
        uint32_t v = kEmptySlot;
        if (j < (uint32_t)a.s && C > 0) { // an empty aggregated neighbourhood samples nothing
            const uint64_t r = bounded64(draw64(rk, j), W);
            int64_t lo = 0, hi = C - 1;
            while (lo < hi) {
                const int64_t mid = lo + ((hi - lo) >> 1);
                if (pre[mid] > r)
                    hi = mid;
                else
                    lo = mid + 1;
            }
            v = (uint32_t)a.p_col[p0 + lo];
        }
        key[j] = v;
    }
    __syncthreads();
    for (uint32_t size = 2; size <= M; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t t = tid; t < (M >> 1); t += 1024) {
                const uint32_t lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                const uint32_t hi = lo | stride;
                const uint32_t x = key[lo], y = key[hi];
                if ((x > y) == ((lo & size) == 0)) {
                    key[lo] = y;
                    key[hi] = x;
                }
            }
            __syncthreads();
        }
    }
    // thread t owns sorted slots [t per, (t+1) per); the first of every run of equal columns stays
    const uint32_t per = M >> 10;
    uint32_t heads = 0;
    for (uint32_t j = tid * per; j < (tid + 1) * per; ++j)
        heads += (key[j] != kEmptySlot && (j == 0 || key[j] != key[j - 1])) ? 1u : 0u;
    uint32_t total;
    uint32_t rank = block_exclusive_scan<uint32_t, 1024>(heads, smem, total);
    int32_t *__restrict__ out = a.sel_tmp + (int64_t)i * a.s;
    for (uint32_t j = tid * per; j < (tid + 1) * per; ++j)
        if (key[j] != kEmptySlot && (j == 0 || key[j] != key[j - 1]))
            out[rank++] = (int32_t)key[j];
    if (tid == 0)
        a.mb_count[i] = total;
}

__global__ __launch_bounds__(256) void ldw_sel_copy_kernel(LwHop a)
{
    const int i = blockIdx.x;
    const int64_t c0 = a.mb_coloff[i], cnt = a.mb_coloff[i + 1] - c0;
    for (int64_t j = threadIdx.x; j < cnt; j += 256)
        a.col_vertex[c0 + j] = a.sel_tmp[(int64_t)i * a.s + j];
}

// ---------------------------------------------------------------------------------------------
// EXTRACT: blockIdx.y = minibatch; the workgroups of a minibatch share its rows wave by wave
// ---------------------------------------------------------------------------------------------
__device__ inline uint32_t ldw_hash(uint32_t v) { return (v * 0x9E3779B1u) >> (32 - 13); }
static_assert(kHashSlots == 1 << 13, "hash width out of step");

__global__ __launch_bounds__(256) void ldw_extract_kernel(LwHop a)
{
    __shared__ uint32_t hkey[kHashSlots];
    __shared__ uint16_t hval[kHashSlots];
    const int i = blockIdx.y, tid = threadIdx.x, lane = tid & (kWave - 1);
    const int64_t c0 = a.mb_coloff[i];
    const int32_t ns = (int32_t)(a.mb_coloff[i + 1] - c0);
    const int64_t r0 = a.mb_rowoff[i], r1 = a.mb_rowoff[i + 1];
    const int64_t wave0 = (int64_t)blockIdx.x * 4 + tid / kWave, nwaves = (int64_t)gridDim.x * 4;
    for (int x = tid; x < kHashSlots; x += 256)
        hkey[x] = kEmptySlot;
    __syncthreads();
    for (int j = tid; j < ns; j += 256) {
        const uint32_t v = (uint32_t)a.col_vertex[c0 + j];
        uint32_t slot = ldw_hash(v);
        while (atomicCAS(&hkey[slot], kEmptySlot, v) != kEmptySlot)
            slot = (slot + 1) & (kHashSlots - 1);
        hval[slot] = (uint16_t)j;
    }
    __syncthreads();
    const uint64_t below = (1ull << lane) - 1ull;
    for (int64_t r = r0 + wave0; r < r1; r += nwaves) {
        const int64_t g0 = a.gather_off[r];
        const uint32_t deg = (uint32_t)(a.gather_off[r + 1] - g0);
        const int32_t *__restrict__ src = a.A_col + a.row_beg[r];
        int32_t *__restrict__ out = a.xtmp + g0;
        uint32_t kept = 0;
        if (ns > 0) {
            for (uint32_t j0 = 0; j0 < deg; j0 += 4 * kWave) {
                uint32_t v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t j = j0 + u * kWave + lane;
                    v[u] = j < deg ? (uint32_t)src[j] : kEmptySlot;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    int32_t local = -1;
                    if (v[u] != kEmptySlot) {
                        uint32_t slot = ldw_hash(v[u]);
                        uint32_t kx;
                        while ((kx = hkey[slot]) != kEmptySlot) {
                            if (kx == v[u]) {
                                local = hval[slot];
                                break;
                            }
                            slot = (slot + 1) & (kHashSlots - 1);
                        }
                    }
                    const uint64_t m = __ballot(local >= 0);
                    if (local >= 0)
                        out[kept + __popcll(m & below)] = local;
                    kept += __popcll(m);
                }
            }
        }
        if (lane == 0)
            a.out_rowptr[r] = kept;
    }
}

// rows to their place: 16 lanes per row
__global__ __launch_bounds__(256) void ldw_extract_copy_kernel(LwHop a)
{
    const int64_t R = a.mb_rowoff[a.k];
    const int sub = threadIdx.x & 15;
    const int64_t groups = (int64_t)gridDim.x * 16;
    for (int64_t r = (int64_t)blockIdx.x * 16 + threadIdx.x / 16; r < R; r += groups) {
        const int64_t o0 = a.out_rowptr[r], cnt = a.out_rowptr[r + 1] - o0;
        const int32_t *__restrict__ src = a.xtmp + a.gather_off[r];
        for (int64_t j = sub; j < cnt; j += 16)
            a.out_col[o0 + j] = src[j];
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
size_t ldw_accumulate_lds_bytes() { return (size_t)(kWinWords + 3 * kAccWaves + 4) * sizeof(uint32_t); }

void launch_ldw_bounds(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_bounds_kernel, dim3(grid_for(L, (a.rows_bound + 3) / 4, 8)), dim3(256), 0, L.stream, a);
}

int launch_ldw_accumulate(const Launch &L, const LwHop &a)
{
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(ldw_accumulate_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldw_accumulate_lds_bytes()) != hipSuccess)
            (void)hipGetLastError(); // not required on every runtime; the launch below reports real failures
        attr_set = true;
    }
    (void)hipMemsetAsync(a.cursor, 0, sizeof(unsigned long long), L.stream);
    hipLaunchKernelGGL(ldw_accumulate_kernel, dim3(grid_for(L, (int64_t)a.k * a.nwin, 1)), dim3(kAccThreads),
                       ldw_accumulate_lds_bytes(), L.stream, a);
    if (hipGetLastError() != hipSuccess)
        return -1;
    hipLaunchKernelGGL(ldw_win_scan_kernel, dim3(a.k), dim3(256), 0, L.stream, a);
    return 0;
}

void launch_ldw_p_copy(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_p_copy_kernel, dim3(grid_for(L, (int64_t)a.k * a.nwin, 8)), dim3(256), 0, L.stream, a);
}

void launch_ldw_draw(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_draw_kernel, dim3(a.k), dim3(1024), 0, L.stream, a);
}

void launch_ldw_sel_copy(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_sel_copy_kernel, dim3(a.k), dim3(256), 0, L.stream, a);
}

void launch_ldw_extract(const Launch &L, const LwHop &a)
{
    int per_mb = (L.num_cu * 8 + a.k - 1) / a.k; // workgroups per minibatch: about 8 per compute unit in all
    if (per_mb > 64)
        per_mb = 64;
    hipLaunchKernelGGL(ldw_extract_kernel, dim3(per_mb, a.k), dim3(256), 0, L.stream, a);
}

void launch_ldw_extract_copy(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_extract_copy_kernel, dim3(grid_for(L, (a.rows_bound + 15) / 16, 8)), dim3(256), 0, L.stream, a);
}

} // namespace bms
