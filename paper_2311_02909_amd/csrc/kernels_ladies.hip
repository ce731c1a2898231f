// Layer-wise (LADIES) bulk sampling kernels, Sec. 4.2 of arxiv 2311.02909.
//
// One hop, all k minibatches at once:
//   ld_rows       extent of every frontier row; exclusive scan of the degrees defines the
//                 "gathered order": the neighbour lists of the stacked frontier laid end to end
//                 (the rows of Q_R A, Sec. 4.2.3)
//   ld_accumulate P = Q A with Q the indicator row of the minibatch's frontier: every gathered
//                 neighbour v adds 1 to the minibatch's dense counter e_v
//   ld_p_*        the nonzero counters compacted in ascending column order -> (p_col, p_cnt)
//   ld_prefix     inclusive prefix sum of the integer weights (e_v or e_v^2) per minibatch
//                 (NORM stays implicit: draws are integers below the row sum)
//   ld_draw       SAMPLE: s draws per minibatch, each the smallest t with prefix[t] > r; the
//                 picked columns' bits are set in the minibatch's vertex set (duplicates merge)
//   (rank)        vertex set ranked -> sampled columns ascending = next frontier
//   ld_extract_*  EXTRACT: second pass over the gathered order keeping the neighbours that are in
//                 the vertex set ((Q_R A) Q_C), relabelled to their rank; rows sized by an
//                 exclusive scan over per-tile counts, so every row stays in ascending order
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

__global__ __launch_bounds__(256) void ld_rows_kernel(LdHop a)
{
    const int64_t R = a.mb_rowoff[a.k];
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < R; r += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = a.row_vertex[r];
        int64_t beg = 0, deg = 0;
        if (v >= 0 && (int64_t)v < a.n) {
            beg = a.A_rowptr[v];
            deg = a.A_rowptr[v + 1] - beg;
        }
        a.row_beg[r] = beg;
        a.gather_off[r] = deg;
        a.row_mb[r] = locate_segment(a.mb_rowoff, a.k, r);
        a.out_rowptr[r] = 0; // per-row counters of the extraction pass
    }
}

__global__ void ld_tiles_kernel(const int64_t *__restrict__ gather_off, const int64_t *__restrict__ R,
                                int64_t *gather_tiles, int64_t *out_rowptr)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *gather_tiles = (gather_off[*R] + kGatherTile - 1) / kGatherTile;
        out_rowptr[*R] = 0;
    }
}

void launch_ld_rows(const Launch &L, const LdHop &a, int64_t *gather_total_out)
{
    hipLaunchKernelGGL(ld_rows_kernel, dim3(grid_for(L, (a.rows_bound + 255) / 256, 8)), dim3(256), 0, L.stream, a);
    launch_scan_i64(L, a.gather_off, a.mb_rowoff + a.k, gather_total_out, nullptr, nullptr, a.rows_bound);
    hipLaunchKernelGGL(ld_tiles_kernel, dim3(1), dim3(64), 0, L.stream, a.gather_off, a.mb_rowoff + a.k,
                       a.gather_tiles, a.out_rowptr);
}

// Walks 16 consecutive positions of the gathered order starting at g0 and calls
// f(q, row, vertex) for position g0 + q (q is a compile-time constant in each call site after
// unrolling, so callers may index register arrays with it).  Empty rows are stepped over.
template <class F>
__device__ inline void for_each_gathered16(const LdHop &a, int64_t g0, int64_t D, int64_t R, F f)
{
    if (g0 >= D)
        return;
    int64_t lo = 0, hi = R; // last row with gather_off[row] <= g0
    while (hi - lo > 1) {
        const int64_t mid = (lo + hi) >> 1;
        if (a.gather_off[mid] <= g0)
            lo = mid;
        else
            hi = mid;
    }
    int64_t r = lo;
    int64_t row_start = a.gather_off[r], row_end = a.gather_off[r + 1];
    const int32_t *__restrict__ src = a.A_col + a.row_beg[r];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int64_t g = g0 + q;
        if (g >= D)
            break;
        if (g >= row_end) {
            do {
                ++r;
                row_end = a.gather_off[r + 1];
            } while (g >= row_end);
            row_start = a.gather_off[r];
            src = a.A_col + a.row_beg[r];
        }
        f(q, r, src[g - row_start]);
    }
}

__global__ __launch_bounds__(256) void ld_accumulate_kernel(LdHop a)
{
    const int64_t R = a.mb_rowoff[a.k];
    const int64_t D = a.gather_off[R];
    const int64_t ntiles = *a.gather_tiles;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t g0 = t * kGatherTile + (int64_t)threadIdx.x * 16;
        for_each_gathered16(a, g0, D, R, [&](int, int64_t r, int32_t v) {
            atomicAdd(&a.counters[(int64_t)a.row_mb[r] * a.n + v], 1u);
        });
    }
}

void launch_ld_accumulate(const Launch &L, const LdHop &a)
{
    hipLaunchKernelGGL(ld_accumulate_kernel, dim3(L.num_cu * 8), dim3(256), 0, L.stream, a);
}

// ---------------------------------------------------------------------------------------------
// Compaction of the dense counters into the sparse row of P (columns ascending).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ld_p_count_kernel(LdHop a)
{
    __shared__ int32_t wsum[4];
    const int64_t nblocks = (int64_t)a.k * a.nchunk;
    for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int64_t i = blk / a.nchunk;
        const int64_t v0 = (blk % a.nchunk) * kPChunk + (int64_t)threadIdx.x * 16;
        const uint32_t *__restrict__ c = a.counters + i * a.n;
        int cnt = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q)
            if (v0 + q < a.n && c[v0 + q] != 0)
                ++cnt;
        cnt = wave_sum(cnt);
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0)
            wsum[threadIdx.x / kWave] = cnt;
        __syncthreads();
        if (threadIdx.x == 0)
            a.p_chunks[blk] = (int64_t)wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
}

void launch_ld_p_count(const Launch &L, const LdHop &a, int64_t *pnnz_out)
{
    hipLaunchKernelGGL(ld_p_count_kernel, dim3(grid_for(L, (int64_t)a.k * a.nchunk, 16)), dim3(256), 0, L.stream, a);
    launch_chunk_scan(L, a.p_chunks, a.k, a.nchunk, a.p_off, pnnz_out);
}

__global__ __launch_bounds__(256) void ld_p_fill_kernel(LdHop a)
{
    __shared__ int32_t smem[4];
    const int64_t nblocks = (int64_t)a.k * a.nchunk;
    for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int64_t i = blk / a.nchunk;
        const int64_t v0 = (blk % a.nchunk) * kPChunk + (int64_t)threadIdx.x * 16;
        const uint32_t *__restrict__ c = a.counters + i * a.n;
        uint32_t val[16];
        int cnt = 0;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            val[q] = (v0 + q < a.n) ? c[v0 + q] : 0u;
            cnt += val[q] != 0;
        }
        int total;
        const int ex = block_exclusive_scan<int32_t, 256>(cnt, smem, total);
        if (cnt) {
            int64_t w = a.p_off[i] + a.p_chunks[blk] + ex;
#pragma unroll
            for (int q = 0; q < 16; ++q)
                if (val[q]) {
                    a.p_col[w] = (int32_t)(v0 + q);
                    a.p_cnt[w] = val[q];
                    ++w;
                }
        }
    }
}

void launch_ld_p_fill(const Launch &L, const LdHop &a)
{
    hipLaunchKernelGGL(ld_p_fill_kernel, dim3(grid_for(L, (int64_t)a.k * a.nchunk, 16)), dim3(256), 0, L.stream, a);
}

// Counters go back to zero by visiting only the nonzero ones (the columns of P).
__global__ __launch_bounds__(256) void ld_clear_counters_kernel(LdHop a)
{
    const int64_t ntiles = a.p_tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(a.p_tileoff, a.k, t);
        const int64_t x0 = a.p_off[i] + (t - a.p_tileoff[i]) * kPTile;
        uint32_t *__restrict__ c = a.counters + (int64_t)i * a.n;
        for (int64_t x = x0 + threadIdx.x; x < x0 + kPTile && x < a.p_off[i + 1]; x += 256)
            c[a.p_col[x]] = 0u;
    }
}

void launch_ld_clear_counters(const Launch &L, const LdHop &a)
{
    hipLaunchKernelGGL(ld_clear_counters_kernel, dim3(grid_for(L, a.pnnz_bound / kPTile + a.k, 8)), dim3(256), 0,
                       L.stream, a);
}

// ---------------------------------------------------------------------------------------------
// Inclusive prefix sums of the weights, restarting at every minibatch.  Tiles of kPTile entries
// never straddle minibatches (p_tileoff): tile sums, per-minibatch scan of them, final pass.
// ---------------------------------------------------------------------------------------------
__device__ inline uint64_t ld_weight(uint32_t cnt, int squared)
{
    return squared ? (uint64_t)cnt * (uint64_t)cnt : (uint64_t)cnt;
}

__global__ __launch_bounds__(256) void ld_prefix_tilesum_kernel(LdHop a)
{
    __shared__ uint64_t wsum[4];
    const int64_t ntiles = a.p_tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(a.p_tileoff, a.k, t);
        const int64_t x0 = a.p_off[i] + (t - a.p_tileoff[i]) * kPTile;
        const int64_t xend = a.p_off[i + 1];
        uint64_t sum = 0;
#pragma unroll
        for (int q = 0; q < kPTile / 256; ++q) {
            const int64_t x = x0 + q * 256 + threadIdx.x;
            if (x < xend)
                sum += ld_weight(a.p_cnt[x], a.squared);
        }
        sum = wave_sum(sum);
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0)
            wsum[threadIdx.x / kWave] = sum;
        __syncthreads();
        if (threadIdx.x == 0)
            a.p_tilesum[t] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
}

// one workgroup per minibatch: exclusive scan of its tile sums in place
__global__ __launch_bounds__(1024) void ld_prefix_tilescan_kernel(LdHop a)
{
    __shared__ uint64_t smem[16];
    __shared__ uint64_t carry_s;
    const int64_t t0 = a.p_tileoff[blockIdx.x], t1 = a.p_tileoff[blockIdx.x + 1];
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (int64_t base = t0; base < t1; base += 1024) {
        const int64_t t = base + threadIdx.x;
        const uint64_t v = t < t1 ? a.p_tilesum[t] : 0;
        uint64_t total;
        const uint64_t ex = block_exclusive_scan<uint64_t, 1024>(v, smem, total);
        const uint64_t carry = carry_s;
        if (t < t1)
            a.p_tilesum[t] = carry + ex;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + total;
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void ld_prefix_fill_kernel(LdHop a)
{
    __shared__ uint64_t smem[4];
    const int64_t ntiles = a.p_tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(a.p_tileoff, a.k, t);
        const int64_t xend = a.p_off[i + 1];
        // each lane owns kPTile/256 consecutive entries
        const int64_t x0 = a.p_off[i] + (t - a.p_tileoff[i]) * kPTile + (int64_t)threadIdx.x * (kPTile / 256);
        uint64_t w[kPTile / 256];
        uint64_t mine = 0;
#pragma unroll
        for (int q = 0; q < kPTile / 256; ++q) {
            w[q] = (x0 + q < xend) ? ld_weight(a.p_cnt[x0 + q], a.squared) : 0;
            mine += w[q];
        }
        uint64_t total;
        uint64_t run = block_exclusive_scan<uint64_t, 256>(mine, smem, total) + a.p_tilesum[t];
#pragma unroll
        for (int q = 0; q < kPTile / 256; ++q) {
            run += w[q];
            if (x0 + q < xend)
                a.prefix[x0 + q] = run;
        }
    }
}

void launch_ld_prefix(const Launch &L, const LdHop &a)
{
    launch_plan_tiles(L, a.p_off, a.k, kPTile, a.p_tileoff);
    const int grid = grid_for(L, a.pnnz_bound / kPTile + a.k, 8);
    hipLaunchKernelGGL(ld_prefix_tilesum_kernel, dim3(grid), dim3(256), 0, L.stream, a);
    hipLaunchKernelGGL(ld_prefix_tilescan_kernel, dim3(a.k), dim3(1024), 0, L.stream, a);
    hipLaunchKernelGGL(ld_prefix_fill_kernel, dim3(grid), dim3(256), 0, L.stream, a);
}

// ---------------------------------------------------------------------------------------------
// SAMPLE (Sec. 4.2.2): draw j of minibatch i is r in [0, W_i); pick the smallest t with
// prefix[t] > r.  One lane per draw.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ld_draw_kernel(LdHop a, VSet vs)
{
    const int64_t total = (int64_t)a.k * a.s;
    for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = x / a.s;
        const uint32_t j = (uint32_t)(x % a.s);
        const int64_t p0 = a.p_off[i], C = a.p_off[i + 1] - p0;
        if (C == 0)
            continue; // empty aggregated neighbourhood: nothing to sample
        const uint64_t *__restrict__ pre = a.prefix + p0;
        const uint64_t W = pre[C - 1];
        const uint64_t key = row_key(a.hopkey, a.mb_base + (uint32_t)i, kNoVertex);
        const uint64_t r = bounded64(draw64(key, j), W);
        int64_t lo = 0, hi = C - 1;
        while (lo < hi) {
            const int64_t mid = lo + ((hi - lo) >> 1);
            if (pre[mid] > r)
                hi = mid;
            else
                lo = mid + 1;
        }
        const int32_t v = a.p_col[p0 + lo];
        atomicOr(&vs.words[i * vs.nw + (v >> 5)], 1u << (v & 31));
    }
}

void launch_ld_draw(const Launch &L, const LdHop &a, const VSet &vs)
{
    hipLaunchKernelGGL(ld_draw_kernel, dim3(grid_for(L, ((int64_t)a.k * a.s + 255) / 256, 8)), dim3(256), 0, L.stream,
                       a, vs);
}

// ---------------------------------------------------------------------------------------------
// EXTRACT (Sec. 4.2.3): keep the gathered neighbours that were sampled.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ld_extract_count_kernel(LdHop a, VSet vs)
{
    __shared__ int32_t wsum[4];
    const int64_t R = a.mb_rowoff[a.k];
    const int64_t D = a.gather_off[R];
    const int64_t ntiles = *a.gather_tiles;
    unsigned long long *rowcnt = reinterpret_cast<unsigned long long *>(a.out_rowptr);
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t g0 = t * kGatherTile + (int64_t)threadIdx.x * 16;
        int mine = 0, run = 0;
        int64_t run_row = -1;
        for_each_gathered16(a, g0, D, R, [&](int, int64_t r, int32_t v) {
            if (r != run_row) {
                if (run)
                    atomicAdd(&rowcnt[run_row], (unsigned long long)run);
                run_row = r;
                run = 0;
            }
            if (vset_test(vs.words + (int64_t)a.row_mb[r] * vs.nw, v)) {
                ++run;
                ++mine;
            }
        });
        if (run)
            atomicAdd(&rowcnt[run_row], (unsigned long long)run);
        mine = wave_sum(mine);
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0)
            wsum[threadIdx.x / kWave] = mine;
        __syncthreads();
        if (threadIdx.x == 0)
            a.tile_off[t] = (int64_t)wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
}

void launch_ld_extract_count(const Launch &L, const LdHop &a, const VSet &vs, int64_t *nnz_out)
{
    hipLaunchKernelGGL(ld_extract_count_kernel, dim3(L.num_cu * 8), dim3(256), 0, L.stream, a, vs);
    launch_scan_i64(L, a.tile_off, a.gather_tiles, nnz_out, nullptr, nullptr);
    launch_scan_i64(L, a.out_rowptr, a.mb_rowoff + a.k, nullptr, nullptr, nullptr);
}

__global__ __launch_bounds__(256) void ld_extract_fill_kernel(LdHop a, VSet vs)
{
    __shared__ int32_t smem[4];
    const int64_t R = a.mb_rowoff[a.k];
    const int64_t D = a.gather_off[R];
    const int64_t ntiles = *a.gather_tiles;
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int64_t g0 = t * kGatherTile + (int64_t)threadIdx.x * 16;
        int32_t kept[16];
        uint32_t mask = 0;
        for_each_gathered16(a, g0, D, R, [&](int q, int64_t r, int32_t v) {
            const int64_t i = a.row_mb[r];
            const uint32_t *__restrict__ words = vs.words + i * vs.nw;
            kept[q] = 0;
            if (vset_test(words, v)) {
                kept[q] = vset_rank_of(words, vs.line_prefix + i * vs.nl, v);
                mask |= 1u << q;
            }
        });
        int total;
        const int ex = block_exclusive_scan<int32_t, 256>(__popc(mask), smem, total);
        int32_t *__restrict__ dst = a.out_col + a.tile_off[t] + ex;
#pragma unroll
        for (int q = 0; q < 16; ++q)
            if (mask & (1u << q))
                *dst++ = kept[q];
    }
}

void launch_ld_extract_fill(const Launch &L, const LdHop &a, const VSet &vs)
{
    hipLaunchKernelGGL(ld_extract_fill_kernel, dim3(L.num_cu * 8), dim3(256), 0, L.stream, a, vs);
}

} // namespace bms
