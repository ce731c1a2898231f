// Node-wise (GraphSAGE) bulk sampling kernels, Sec. 4.1 of arxiv 2311.02909.
//
// One hop over the stacked frontier (all k minibatches at once, Eq. 1):
//   nw_rows    P = Q A: Q has one nonzero per row, so row r of P is the CSR row of the frontier
//              vertex; only its extent (begin, degree) is fetched.  Also the per-tile sums of
//              min(degree, s) that size the output rows.
//   (scan)     exclusive scan of the tile sums -> where each tile's output starts
//   nw_sample  SAMPLE: per row, min(degree, s) distinct positions (ITS without replacement,
//              Sec. 4.1.2), the chosen neighbours gathered, staged through LDS and written
//              coalesced as global ids
// EXTRACT (Sec. 4.1.3: distinct sampled ids ascending = next frontier, global id -> local column) is
// done by the kernels of kernels_dedup_sort.hip / kernels_dedup.hip.  The first design of it lives
// here and serves vertex ranges too wide for those: nw_sample also sets the ids' bits in a
// per-minibatch vertex set in HBM, the set is ranked (kernels_common.hip), and
//   nw_relabel global id -> local column index = rank in the minibatch's vertex set
// Variant (the frontier's own vertices stay columns): every row carries its own vertex as one more
// entry through EXTRACT, and nw_strip_self takes it out of the row again afterwards.
// Variant (independent draws): the s draws of a row are each an integer in [0, degree), the row keeps
// the distinct picks; its length is only known after the draws, so nw_rows makes them too.
#include "bms_device.h"
#include "bms_internal.h"

#include <algorithm>

namespace bms {

// Independent draws (ITS with replacement on the unit weights of a row): s integers in [0, deg), kept sorted
// in c[0..s) by one bubble pass per draw.  Returns the number of distinct values.
template <int S>
__device__ __forceinline__ int32_t replace_draws(uint64_t key, uint32_t deg, int32_t s, uint32_t (&c)[S])
{
#pragma unroll
    for (int j = 0; j < S; ++j) {
        if (j < s) {
            c[j] = bounded32(draw32(key, (uint32_t)j), deg);
#pragma unroll
            for (int q = j; q > 0; --q) {
                const uint32_t lo = min(c[q - 1], c[q]);
                const uint32_t hi = max(c[q - 1], c[q]);
                c[q - 1] = lo;
                c[q] = hi;
            }
        }
    }
    int32_t m = 0;
#pragma unroll
    for (int j = 0; j < S; ++j)
        if (j < s)
            m += (j == 0 || c[j] != c[j - 1]) ? 1 : 0;
    return m;
}

// The same for any s <= kMaxSampledFanout by one wave: the draws are written to `buf` (LDS, room for the next
// power of two >= max(s, 64)), sorted there by a bitonic network, and the distinct values moved down to
// buf[0..m) in ascending order.  Returns m (the same value in every lane).
__device__ inline int32_t wave_replace_draws(volatile uint32_t *buf, uint64_t key, uint32_t deg, int32_t s, int lane)
{
    int32_t P = kWave;
    while (P < s)
        P <<= 1;
    for (int32_t j = lane; j < P; j += kWave)
        buf[j] = j < s ? bounded32(draw32(key, (uint32_t)j), deg) : 0xFFFFFFFFu; // padding sorts last (deg < 2^31)
    __builtin_amdgcn_wave_barrier();
    for (int32_t size = 2; size <= P; size <<= 1) {
        for (int32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (int32_t t = lane; t < P / 2; t += kWave) {
                const int32_t lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1)); // bit `stride` clear
                const int32_t hi = lo | stride;
                const bool up = (lo & size) == 0;
                const uint32_t x = buf[lo], y = buf[hi];
                if ((x > y) == up) {
                    buf[lo] = y;
                    buf[hi] = x;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    int32_t m = 0;
    uint32_t last = 0; // value before this chunk's first one
    for (int32_t base = 0; base < P; base += kWave) {
        const int32_t j = base + lane;
        const uint32_t v = buf[j];
        uint32_t prev = __shfl_up(v, 1);
        if (lane == 0)
            prev = last;
        const bool head = j < s && (j == 0 || v != prev);
        const uint64_t heads = __ballot(head);
        __builtin_amdgcn_wave_barrier(); // the chunk is read before any of it is overwritten (targets are <= sources)
        if (head)
            buf[m + __popcll(heads & ((1ull << lane) - 1ull))] = v;
        m += __popcll(heads);
        last = __shfl(v, kWave - 1);
        __builtin_amdgcn_wave_barrier();
    }
    return m;
}

// S = 0: rows keep min(degree, s) entries.  S > 0: independent draws, s <= S; the row's length is the number
// of distinct picks.
template <int S>
__global__ __launch_bounds__(kRowTile) void nw_rows_kernel(NwHop a)
{
    __shared__ int64_t wsum[kRowTile / kWave];
    const int tid = threadIdx.x;
    // Tile j of every minibatch before tile j + 1 of any: the rows of a minibatch ascend by vertex id, so the
    // workgroups that run at the same time touch the same part of the id range in all minibatches, and lines of
    // rowptr / col that several minibatches need are still in the last-level cache when the next one asks.
    const int64_t most = a.mb_tileoff[a.k + 1]; // tiles of the minibatch that has most
    for (int64_t v = blockIdx.x; v < most * a.k; v += gridDim.x) {
        const int i = (int)(v % a.k);
        const int64_t j = v / a.k;
        if (j >= a.mb_tileoff[i + 1] - a.mb_tileoff[i])
            continue;
        const int64_t t = a.mb_tileoff[i] + j;
        const int64_t r = a.mb_rowoff[i] + j * kRowTile + tid;
        int64_t cnt = 0;
        if (r < a.mb_rowoff[i + 1]) {
            const int32_t v = a.row_vertex[r];
            int64_t beg = 0, deg = 0;
            if (v >= 0 && (int64_t)v < a.n) { // seeds are verified separately; never read out of bounds
                beg = a.A_rowptr[v];
                deg = a.A_rowptr[v + 1] - beg;
            }
            a.row_beg[r] = beg;
            a.row_deg[r] = (int32_t)deg;
            if (S == 0) {
                cnt = deg < a.s ? deg : a.s;
            } else if (deg > 0) {
                uint32_t c[S > 0 ? S : 1];
                cnt = replace_draws(row_key(a.hopkey, a.mb_base + (uint32_t)i, (uint32_t)v), (uint32_t)deg, a.s, c);
            }
            cnt += a.self_entry;
        }
        cnt = wave_sum(cnt);
        __syncthreads();
        if ((tid & (kWave - 1)) == 0)
            wsum[tid / kWave] = cnt;
        __syncthreads();
        if (tid == 0) {
            int64_t tot = 0;
#pragma unroll
            for (int w = 0; w < kRowTile / kWave; ++w)
                tot += wsum[w];
            a.tile_off[t] = tot;
        }
    }
}

// Independent draws with s > 32: extents by one row per lane as above, then one row per wave: draws sorted in
// LDS, distinct ones counted; the count is kept per row (row_cnt) so that the sampling kernel can place the
// rows before it repeats the draws.
__global__ __launch_bounds__(kRowTile) void nw_rows_replace_wide_kernel(NwHop a)
{
    __shared__ uint32_t chosen_all[(kRowTile / kWave) * kMaxSampledFanout];
    __shared__ int64_t wsum[kRowTile / kWave];
    __shared__ int32_t deg_of[kRowTile], vert_of[kRowTile], cnt_of[kRowTile];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    volatile uint32_t *buf = chosen_all + wave * kMaxSampledFanout;
    const int64_t most = a.mb_tileoff[a.k + 1];
    for (int64_t v = blockIdx.x; v < most * a.k; v += gridDim.x) {
        const int i = (int)(v % a.k);
        const int64_t j = v / a.k;
        if (j >= a.mb_tileoff[i + 1] - a.mb_tileoff[i])
            continue;
        const int64_t t = a.mb_tileoff[i] + j;
        const int64_t r0 = a.mb_rowoff[i] + j * kRowTile;
        const int64_t r = r0 + tid;
        const int64_t left = a.mb_rowoff[i + 1] - r0;
        const int nr = (int)(left < kRowTile ? left : kRowTile);
        if (tid < nr) {
            const int32_t vtx = a.row_vertex[r];
            int64_t beg = 0, deg = 0;
            if (vtx >= 0 && (int64_t)vtx < a.n) {
                beg = a.A_rowptr[vtx];
                deg = a.A_rowptr[vtx + 1] - beg;
            }
            a.row_beg[r] = beg;
            a.row_deg[r] = (int32_t)deg;
            deg_of[tid] = (int32_t)deg;
            vert_of[tid] = vtx;
        }
        __syncthreads();
        for (int q = wave; q < nr; q += kRowTile / kWave) {
            int32_t m = 0;
            if (deg_of[q] > 0)
                m = wave_replace_draws(buf, row_key(a.hopkey, a.mb_base + (uint32_t)i, (uint32_t)vert_of[q]),
                                       (uint32_t)deg_of[q], a.s, lane);
            if (lane == 0)
                cnt_of[q] = m;
        }
        __syncthreads();
        int64_t cnt = 0;
        if (tid < nr) {
            a.row_cnt[r] = cnt_of[tid];
            cnt = cnt_of[tid] + a.self_entry;
        }
        cnt = wave_sum(cnt);
        if (lane == 0)
            wsum[wave] = cnt;
        __syncthreads();
        if (tid == 0) {
            int64_t tot = 0;
#pragma unroll
            for (int w = 0; w < kRowTile / kWave; ++w)
                tot += wsum[w];
            a.tile_off[t] = tot;
        }
        __syncthreads();
    }
}

void launch_nw_rows(const Launch &L, const NwHop &a)
{
    const int64_t tiles = a.rows_bound / kRowTile + a.k;
    const dim3 grid(grid_for(L, tiles, 16)), block(kRowTile);
    if (!a.replace)
        hipLaunchKernelGGL(nw_rows_kernel<0>, grid, block, 0, L.stream, a);
    else if (a.s <= 4)
        hipLaunchKernelGGL(nw_rows_kernel<4>, grid, block, 0, L.stream, a);
    else if (a.s <= 8)
        hipLaunchKernelGGL(nw_rows_kernel<8>, grid, block, 0, L.stream, a);
    else if (a.s <= 16)
        hipLaunchKernelGGL(nw_rows_kernel<16>, grid, block, 0, L.stream, a);
    else if (a.s <= 32)
        hipLaunchKernelGGL(nw_rows_kernel<32>, grid, block, 0, L.stream, a);
    else
        hipLaunchKernelGGL(nw_rows_replace_wide_kernel, dim3(grid_for(L, tiles, 2)), block, 0, L.stream, a);
}

// ---------------------------------------------------------------------------------------------
// SAMPLE, one row per lane, fanout <= S (compile-time capacity of the per-lane position list).
//
// Without-replacement rule: draw j is an integer x in [0, deg - j), the index of the pick among
// the positions not chosen so far in ascending order (inverse-transform sampling on the unit
// weights with the chosen entries zeroed).  Stepping x over every chosen position <= x, in
// ascending order, turns it into the position; the list is kept sorted by one bubble pass,
// which also leaves the row's output in ascending column order.
// ---------------------------------------------------------------------------------------------
template <int S, bool SET, bool REPLACE>
__global__ __launch_bounds__(kRowTile) void nw_sample_kernel(NwHop a, VSet vs)
{
    __shared__ int32_t stage[kRowTile * (S + 1)]; // + 1: the row's own vertex when rows carry it
    __shared__ int32_t wsum[kRowTile / kWave];
    __shared__ uint32_t seg_hist[kMaxFusedSegments]; // sampled ids per id-range segment, of this workgroup's minibatch
    __shared__ uint16_t seg_tab_l[kMaxCells + 1];    // segment of every cell of ids, when the segments differ in width
    const int tid = threadIdx.x;
    const int64_t most = a.mb_tileoff[a.k + 1];
    const int32_t s = a.s;
    const bool count = a.seg_cnt != nullptr; // then gridDim.x is a multiple of k: every tile of this workgroup belongs
                                             // to minibatch blockIdx.x % k
    const bool by_table = count && a.seg_tab != nullptr;
    if (count) {
        for (int c = tid; c < a.seg_C; c += kRowTile)
            seg_hist[c] = 0;
        if (by_table)
            for (int x = tid; x <= kMaxCells; x += kRowTile)
                seg_tab_l[x] = a.seg_tab[x];
        __syncthreads();
    }
    // the extent of the lane's row in the workgroup's next tile is fetched while the current tile is sampled
    auto extent = [&](int64_t v, int64_t &beg, int32_t &deg) {
        beg = 0;
        deg = 0;
        if (v < most * a.k) {
            const int i = (int)(v % a.k);
            const int64_t j = v / a.k;
            const int64_t r = a.mb_rowoff[i] + j * kRowTile + tid;
            if (j < a.mb_tileoff[i + 1] - a.mb_tileoff[i] && r < a.mb_rowoff[i + 1]) {
                beg = a.row_beg[r];
                deg = a.row_deg[r];
            }
        }
    };
    int64_t beg, beg_next;
    int32_t deg, deg_next;
    extent(blockIdx.x, beg, deg);
    for (int64_t v = blockIdx.x; v < most * a.k; v += gridDim.x, beg = beg_next, deg = deg_next) { // same order as nw_rows_kernel
        extent(v + gridDim.x, beg_next, deg_next);
        const int i = (int)(v % a.k);
        const int64_t j = v / a.k;
        if (j >= a.mb_tileoff[i + 1] - a.mb_tileoff[i])
            continue;
        const int64_t t = a.mb_tileoff[i] + j;
        const int64_t r = a.mb_rowoff[i] + j * kRowTile + tid;
        const bool valid = r < a.mb_rowoff[i + 1];
        int32_t cnt = 0;
        uint32_t c[S];
        if (valid) {
            if (!REPLACE)
                cnt = deg < s ? deg : s;
            else if (deg > 0) // independent draws: the row's length is the number of distinct picks
                cnt = replace_draws(row_key(a.hopkey, a.mb_base + (uint32_t)i, (uint32_t)a.row_vertex[r]),
                                    (uint32_t)deg, s, c);
        }
        int32_t tot;
        const int32_t loc = block_exclusive_scan<int32_t, kRowTile>(valid ? cnt + a.self_entry : 0, wsum, tot);
        const int64_t base = a.tile_off[t];
        if (valid)
            a.out_rowptr[r] = base + loc;
        if (valid && a.self_entry) { // a seed outside [0, n) is reported by the seed check; EXTRACT still gets a valid id
            const int32_t self = a.row_vertex[r];
            stage[loc + cnt] = (self >= 0 && (int64_t)self < a.n) ? self : 0;
        }
        if (REPLACE) {
            if (cnt > 0) {
                const int32_t *__restrict__ src = a.A_col + beg;
                int32_t m = 0;
#pragma unroll
                for (int j = 0; j < S; ++j)
                    if (j < s && (j == 0 || c[j] != c[j - 1]))
                        stage[loc + m++] = src[c[j]];
            }
        } else if (cnt > 0) {
            if (deg <= s) {
#pragma unroll
                for (int j = 0; j < S; ++j)
                    c[j] = (uint32_t)j;
            } else {
                const uint64_t key = row_key(a.hopkey, a.mb_base + (uint32_t)i, (uint32_t)a.row_vertex[r]);
#pragma unroll
                for (int j = 0; j < S; ++j) {
                    if (j < s) {
                        uint32_t x = bounded32(draw32(key, (uint32_t)j), (uint32_t)deg - (uint32_t)j);
#pragma unroll
                        for (int q = 0; q < j; ++q)
                            x += (x >= c[q]) ? 1u : 0u;
                        c[j] = x;
#pragma unroll
                        for (int q = j; q > 0; --q) {
                            const uint32_t lo = min(c[q - 1], c[q]);
                            const uint32_t hi = max(c[q - 1], c[q]);
                            c[q - 1] = lo;
                            c[q] = hi;
                        }
                    }
                }
            }
            const int32_t *__restrict__ src = a.A_col + beg;
#pragma unroll
            for (int j = 0; j < S; ++j)
                if (j < cnt)
                    stage[loc + j] = src[c[j]];
        }
        __syncthreads();
        uint32_t *__restrict__ words = vs.words + (int64_t)i * vs.nw;
        for (int32_t e = tid; e < tot; e += kRowTile) {
            const int32_t g = stage[e];
            a.out_col[base + e] = g;
            if (SET)
                atomicOr(&words[g >> 5], 1u << (g & 31));
            if (count)
                atomicAdd(&seg_hist[by_table ? (uint32_t)seg_tab_l[(uint32_t)g >> a.seg_shift] : (uint32_t)g >> a.seg_shift], 1u);
        }
        __syncthreads();
    }
    if (count) {
        uint32_t *__restrict__ out = a.seg_cnt + (int64_t)(blockIdx.x % a.k) * a.seg_C;
        for (int c = tid; c < a.seg_C; c += kRowTile)
            if (seg_hist[c])
                atomicAdd(&out[c], seg_hist[c]);
    }
}

// ---------------------------------------------------------------------------------------------
// SAMPLE, one row per wave, any fanout: rows with degree <= s are copied whole; longer rows keep
// their sorted chosen list in LDS (s <= kMaxSampledFanout).  For draw j the number c of chosen
// positions that the pick steps over is the count of list entries p_t with p_t - t <= x
// (p_t - t = unchosen positions before p_t, non-decreasing in t), found by binary search.
// ---------------------------------------------------------------------------------------------
template <bool SET, bool REPLACE>
__global__ __launch_bounds__(kRowTile) void nw_sample_wide_kernel(NwHop a, VSet vs)
{
    __shared__ uint32_t chosen_all[(kRowTile / kWave) * kMaxSampledFanout];
    __shared__ int64_t wsum[kRowTile / kWave];
    __shared__ int64_t row_loc[kRowTile];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    volatile uint32_t *chosen = chosen_all + wave * kMaxSampledFanout;
    const int64_t ntiles = a.mb_tileoff[a.k];
    const int32_t s = a.s;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(a.mb_tileoff, a.k, t);
        const int64_t r0 = a.mb_rowoff[i] + (t - a.mb_tileoff[i]) * kRowTile;
        const int64_t rend = a.mb_rowoff[i + 1];
        const int64_t r = r0 + tid;
        int64_t cnt = 0;
        if (r < rend) {
            const int64_t deg = a.row_deg[r];
            cnt = (REPLACE ? (int64_t)a.row_cnt[r] : (deg < s ? deg : s)) + a.self_entry;
        }
        int64_t tot;
        const int64_t loc = block_exclusive_scan<int64_t, kRowTile>(cnt, wsum, tot);
        const int64_t base = a.tile_off[t];
        if (r < rend)
            a.out_rowptr[r] = base + loc;
        row_loc[tid] = base + loc;
        __syncthreads();
        uint32_t *__restrict__ words = vs.words + (int64_t)i * vs.nw;
        for (int q = wave; q < kRowTile; q += kRowTile / kWave) { // rows of this tile, one per wave
            const int64_t rr = r0 + q;
            if (rr >= rend)
                break;
            const int64_t beg = a.row_beg[rr];
            const int32_t deg = a.row_deg[rr];
            int32_t *__restrict__ dst = a.out_col + row_loc[q];
            const int32_t *__restrict__ src = a.A_col + beg;
            if (a.self_entry && lane == 0) { // the row's own vertex, after its sampled ones (kept inside [0, n):
                                             // a bad seed is reported by the seed check, EXTRACT still gets a valid id)
                int32_t g = a.row_vertex[rr];
                if (g < 0 || (int64_t)g >= a.n)
                    g = 0;
                dst[REPLACE ? a.row_cnt[rr] : (deg < s ? deg : s)] = g;
                if (SET)
                    atomicOr(&words[g >> 5], 1u << (g & 31));
            }
            if (REPLACE) { // independent draws: the distinct picks, sorted by the wave in LDS
                if (deg > 0) {
                    const int32_t m = wave_replace_draws(
                        chosen, row_key(a.hopkey, a.mb_base + (uint32_t)i, (uint32_t)a.row_vertex[rr]), (uint32_t)deg, s,
                        lane);
                    for (int32_t e = lane; e < m; e += kWave) {
                        const int32_t g = src[chosen[e]];
                        dst[e] = g;
                        if (SET)
                            atomicOr(&words[g >> 5], 1u << (g & 31));
                    }
                    __builtin_amdgcn_wave_barrier();
                }
                continue;
            }
            if (deg <= s) {
                for (int32_t e = lane; e < deg; e += kWave) {
                    const int32_t g = src[e];
                    dst[e] = g;
                    if (SET)
                        atomicOr(&words[g >> 5], 1u << (g & 31));
                }
                continue;
            }
            const uint64_t key = row_key(a.hopkey, a.mb_base + (uint32_t)i, (uint32_t)a.row_vertex[rr]);
            for (int32_t j = 0; j < s; ++j) {
                const uint32_t x = bounded32(draw32(key, (uint32_t)j), (uint32_t)deg - (uint32_t)j);
                // c = number of t in [0,j) with chosen[t] - t <= x   (all lanes compute the same value)
                int32_t lo = 0, hi = j;
                while (lo < hi) {
                    const int32_t mid = (lo + hi) >> 1;
                    if (chosen[mid] - (uint32_t)mid <= x)
                        lo = mid + 1;
                    else
                        hi = mid;
                }
                const int32_t c = lo;
                // shift chosen[c..j) up by one, top chunk first so nothing is overwritten before it is read
                for (int32_t top = j; top > c; top -= kWave) {
                    const int32_t idx = top - 1 - lane; // source index
                    uint32_t val = 0;
                    if (idx >= c)
                        val = chosen[idx];
                    __builtin_amdgcn_wave_barrier();
                    if (idx >= c)
                        chosen[idx + 1] = val;
                    __builtin_amdgcn_wave_barrier();
                }
                if (lane == 0)
                    chosen[c] = x + (uint32_t)c;
                __builtin_amdgcn_wave_barrier();
            }
            for (int32_t e = lane; e < s; e += kWave) {
                const int32_t g = src[chosen[e]];
                dst[e] = g;
                if (SET)
                    atomicOr(&words[g >> 5], 1u << (g & 31));
            }
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();
    }
}

template <bool SET, bool REPLACE>
static bool launch_nw_sample_impl(const Launch &L, const NwHop &a_in, const VSet &vs)
{
    NwHop a = a_in;
    const int64_t tiles = a.rows_bound / kRowTile + a.k;
    if (a.s > 32) {
        a.seg_cnt = nullptr; // one row per wave: its workgroups walk the tiles in stacked order, across minibatches
        hipLaunchKernelGGL((nw_sample_wide_kernel<SET, REPLACE>), dim3(grid_for(L, tiles, 2)), dim3(kRowTile), 0, L.stream, a, vs);
        return false;
    }
    int grid = grid_for(L, tiles, a.s <= 16 ? 8 : 4);
    // counting per segment needs every workgroup to stay with one minibatch: tile v belongs to minibatch v % k,
    // so a grid that is a multiple of k does it
    if (a.seg_cnt && a.seg_C <= kMaxFusedSegments && a.k <= L.num_cu * (a.s <= 16 ? 8 : 4))
        grid = std::max(grid / a.k, 1) * a.k;
    else
        a.seg_cnt = nullptr;
    if (a.s <= 4)
        hipLaunchKernelGGL((nw_sample_kernel<4, SET, REPLACE>), dim3(grid), dim3(kRowTile), 0, L.stream, a, vs);
    else if (a.s <= 8)
        hipLaunchKernelGGL((nw_sample_kernel<8, SET, REPLACE>), dim3(grid), dim3(kRowTile), 0, L.stream, a, vs);
    else if (a.s <= 16)
        hipLaunchKernelGGL((nw_sample_kernel<16, SET, REPLACE>), dim3(grid), dim3(kRowTile), 0, L.stream, a, vs);
    else
        hipLaunchKernelGGL((nw_sample_kernel<32, SET, REPLACE>), dim3(grid), dim3(kRowTile), 0, L.stream, a, vs);
    return a.seg_cnt != nullptr;
}

bool launch_nw_sample(const Launch &L, const NwHop &a, const VSet &vs, bool set_bits)
{
    if (a.replace) {
        if (set_bits)
            return launch_nw_sample_impl<true, true>(L, a, vs);
        return launch_nw_sample_impl<false, true>(L, a, vs);
    }
    if (set_bits)
        return launch_nw_sample_impl<true, false>(L, a, vs);
    return launch_nw_sample_impl<false, false>(L, a, vs);
}

// ---------------------------------------------------------------------------------------------
// EXTRACT: "remove empty columns" -- the kept columns of a minibatch are its set vertices in
// ascending order, so a sampled vertex's local column is its rank in the vertex set:
// line_prefix[line] + set bits before it inside its 64-byte line.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void nw_relabel_kernel(NwHop a, VSet vs)
{
    const int64_t ntiles = a.mb_tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(a.mb_tileoff, a.k, t);
        const uint32_t *__restrict__ words = vs.words + (int64_t)i * vs.nw;
        const uint32_t *__restrict__ prefix = vs.line_prefix + (int64_t)i * vs.nl;
        const int64_t e1 = a.tile_off[t + 1];
        for (int64_t e = a.tile_off[t] + threadIdx.x; e < e1; e += 256)
            a.out_col[e] = vset_rank_of(words, prefix, a.out_col[e]);
    }
}

// ---------------------------------------------------------------------------------------------
// Rows that carried their own vertex through EXTRACT as a trailing entry (so that it became a column
// and got a local index like any sampled vertex): the entry leaves the row again.  Row r loses one
// entry and every row before it one each, so its entries move r places down; the trailing entry is
// the row's own column.  One tile of kRowTile stacked rows per iteration, one entry per lane per
// step, the entry's row found in the tile's row offsets held in LDS.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kRowTile) void nw_strip_self_kernel(const int64_t *__restrict__ rowptr_in,
                                                                 const int32_t *__restrict__ col_in,
                                                                 const int64_t *__restrict__ rows_ptr,
                                                                 int64_t *__restrict__ rowptr_out,
                                                                 int32_t *__restrict__ col_out,
                                                                 int32_t *__restrict__ row_self,
                                                                 int64_t *__restrict__ nnz_slot)
{
    constexpr int kMapCap = kRowTile * 33; // entries of a tile whose rows hold at most 32 sampled vertices
    __shared__ int64_t off[kRowTile + 1];
    __shared__ uint8_t row_of[kMapCap];
    const int tid = threadIdx.x;
    const int64_t rows = *rows_ptr;
    const int64_t ntiles = (rows + kRowTile - 1) / kRowTile;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t r0 = t * kRowTile;
        const int nr = (int)(rows - r0 < kRowTile ? rows - r0 : kRowTile);
        const int64_t e0 = rowptr_in[r0];
        if (tid < nr) {
            const int64_t p = rowptr_in[r0 + tid];
            off[tid] = p - e0;
            rowptr_out[r0 + tid] = p - (r0 + tid);
        }
        if (tid == 0)
            off[nr] = rowptr_in[r0 + nr] - e0;
        __syncthreads();
        const int64_t span = off[nr];
        const bool mapped = span <= kMapCap; // the usual case: every row writes its index over its entries
        if (mapped && tid < nr) {
            const int32_t b = (int32_t)off[tid], e = (int32_t)off[tid + 1];
            for (int32_t q = b; q < e; ++q)
                row_of[q] = (uint8_t)tid;
        }
        if (mapped)
            __syncthreads();
        for (int64_t e = tid; e < span; e += kRowTile) {
            int lo;
            if (mapped) {
                lo = row_of[e];
            } else { // last row with off[row] <= e (rows are never empty: each has its own entry)
                lo = 0;
                int hi = nr;
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (off[mid] <= e)
                        lo = mid;
                    else
                        hi = mid;
                }
            }
            const int32_t g = col_in[e0 + e];
            if (e == off[lo + 1] - 1)
                row_self[r0 + lo] = g;
            else
                col_out[e0 + e - (r0 + lo)] = g;
        }
        __syncthreads();
    }
    if (blockIdx.x == 0 && tid == 0) {
        const int64_t total = rowptr_in[rows];
        rowptr_out[rows] = total - rows;
        *nnz_slot = total - rows;
    }
}

void launch_nw_strip_self(const Launch &L, const int64_t *rowptr_in, const int32_t *col_in, const int64_t *rows,
                          int64_t rows_bound, int64_t *rowptr_out, int32_t *col_out, int32_t *row_self,
                          int64_t *nnz_slot)
{
    const int64_t tiles = rows_bound / kRowTile + 1;
    hipLaunchKernelGGL(nw_strip_self_kernel, dim3(grid_for(L, tiles, 8)), dim3(kRowTile), 0, L.stream, rowptr_in,
                       col_in, rows, rowptr_out, col_out, row_self, nnz_slot);
}

void launch_nw_relabel(const Launch &L, const NwHop &a, const VSet &vs)
{
    const int64_t tiles = a.rows_bound / kRowTile + a.k;
    hipLaunchKernelGGL(nw_relabel_kernel, dim3(grid_for(L, tiles, 16)), dim3(256), 0, L.stream, a, vs);
}

} // namespace bms
