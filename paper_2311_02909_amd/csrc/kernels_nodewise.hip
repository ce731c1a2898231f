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
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

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
            cnt = (deg < a.s ? deg : a.s) + a.self_entry;
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

void launch_nw_rows(const Launch &L, const NwHop &a)
{
    const int64_t tiles = a.rows_bound / kRowTile + a.k;
    hipLaunchKernelGGL(nw_rows_kernel, dim3(grid_for(L, tiles, 16)), dim3(kRowTile), 0, L.stream, a);
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
template <int S, bool SET>
__global__ __launch_bounds__(kRowTile) void nw_sample_kernel(NwHop a, VSet vs)
{
    __shared__ int32_t stage[kRowTile * (S + 1)]; // + 1: the row's own vertex when rows carry it
    __shared__ int32_t wsum[kRowTile / kWave];
    const int tid = threadIdx.x;
    const int64_t most = a.mb_tileoff[a.k + 1];
    const int32_t s = a.s;
    for (int64_t v = blockIdx.x; v < most * a.k; v += gridDim.x) { // same order as nw_rows_kernel
        const int i = (int)(v % a.k);
        const int64_t j = v / a.k;
        if (j >= a.mb_tileoff[i + 1] - a.mb_tileoff[i])
            continue;
        const int64_t t = a.mb_tileoff[i] + j;
        const int64_t r = a.mb_rowoff[i] + j * kRowTile + tid;
        const bool valid = r < a.mb_rowoff[i + 1];
        int64_t beg = 0;
        int32_t deg = 0, cnt = 0;
        if (valid) {
            beg = a.row_beg[r];
            deg = a.row_deg[r];
            cnt = deg < s ? deg : s;
        }
        int32_t tot;
        const int32_t loc = block_exclusive_scan<int32_t, kRowTile>(valid ? cnt + a.self_entry : 0, wsum, tot);
        const int64_t base = a.tile_off[t];
        if (valid)
            a.out_rowptr[r] = base + loc;
        if (valid && a.self_entry)
            stage[loc + cnt] = a.row_vertex[r];
        if (cnt > 0) {
            uint32_t c[S];
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
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// SAMPLE, one row per wave, any fanout: rows with degree <= s are copied whole; longer rows keep
// their sorted chosen list in LDS (s <= kMaxSampledFanout).  For draw j the number c of chosen
// positions that the pick steps over is the count of list entries p_t with p_t - t <= x
// (p_t - t = unchosen positions before p_t, non-decreasing in t), found by binary search.
// ---------------------------------------------------------------------------------------------
template <bool SET>
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
            cnt = (deg < s ? deg : s) + a.self_entry;
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
            if (a.self_entry && lane == 0) { // the row's own vertex, after its min(deg, s) sampled ones
                const int32_t g = a.row_vertex[rr];
                dst[deg < s ? deg : s] = g;
                if (SET)
                    atomicOr(&words[g >> 5], 1u << (g & 31));
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

template <bool SET>
static void launch_nw_sample_impl(const Launch &L, const NwHop &a, const VSet &vs)
{
    const int64_t tiles = a.rows_bound / kRowTile + a.k;
    if (a.s <= 4)
        hipLaunchKernelGGL((nw_sample_kernel<4, SET>), dim3(grid_for(L, tiles, 8)), dim3(kRowTile), 0, L.stream, a, vs);
    else if (a.s <= 8)
        hipLaunchKernelGGL((nw_sample_kernel<8, SET>), dim3(grid_for(L, tiles, 8)), dim3(kRowTile), 0, L.stream, a, vs);
    else if (a.s <= 16)
        hipLaunchKernelGGL((nw_sample_kernel<16, SET>), dim3(grid_for(L, tiles, 8)), dim3(kRowTile), 0, L.stream, a, vs);
    else if (a.s <= 32)
        hipLaunchKernelGGL((nw_sample_kernel<32, SET>), dim3(grid_for(L, tiles, 4)), dim3(kRowTile), 0, L.stream, a, vs);
    else
        hipLaunchKernelGGL((nw_sample_wide_kernel<SET>), dim3(grid_for(L, tiles, 2)), dim3(kRowTile), 0, L.stream, a, vs);
}

void launch_nw_sample(const Launch &L, const NwHop &a, const VSet &vs, bool set_bits)
{
    if (set_bits)
        launch_nw_sample_impl<true>(L, a, vs);
    else
        launch_nw_sample_impl<false>(L, a, vs);
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
