// Kernels shared by both samplers: CSR verification, seed verification, tile planning,
// device-length scans and the per-minibatch vertex set (bitmap + rank).
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

int grid_for(const Launch &L, int64_t blocks, int per_cu)
{
    int64_t cap = (int64_t)L.num_cu * per_cu;
    if (blocks < 1)
        blocks = 1;
    return (int)(blocks < cap ? blocks : cap);
}

// ---------------------------------------------------------------------------------------------
// CSR verification at load time.  flag bit 0: rowptr not monotone / wrong ends, bit 1: column out
// of range, bit 2: row not strictly ascending.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void csr_check_rows_kernel(const int64_t *__restrict__ rowptr, int64_t n, int64_t nnz,
                                                             int32_t *flag, unsigned long long *maxdeg)
{
    __shared__ unsigned long long smax[4];
    unsigned long long best = 0;
    int bad = 0;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
        const int64_t a = rowptr[v], b = rowptr[v + 1];
        if (a > b || a < 0 || b > nnz)
            bad = 1;
        else if ((unsigned long long)(b - a) > best)
            best = (unsigned long long)(b - a);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && (rowptr[0] != 0 || rowptr[n] != nnz))
        bad = 1;
    if (bad)
        atomicOr(flag, 1);
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        unsigned long long o = __shfl_xor(best, d, kWave);
        best = o > best ? o : best;
    }
    if ((threadIdx.x & (kWave - 1)) == 0)
        smax[threadIdx.x / kWave] = best;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 4; ++w)
            best = smax[w] > best ? smax[w] : best;
        if (best)
            atomicMax(maxdeg, best);
    }
}

// One lane per nonzero.  A descent col[e-1] >= col[e] is legal only where a row starts at e,
// which is looked up in rowptr (only evaluated at descents, i.e. about once per row).
__global__ __launch_bounds__(256) void csr_check_cols_kernel(const int64_t *__restrict__ rowptr,
                                                             const int32_t *__restrict__ col, int64_t n, int64_t nnz,
                                                             int32_t *flag)
{
    int bad = 0;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < nnz; e += (int64_t)gridDim.x * blockDim.x) {
        const int32_t c = col[e];
        if (c < 0 || (int64_t)c >= n)
            bad |= 2;
        if (e > 0 && col[e - 1] >= c) {
            // first row index v with rowptr[v] >= e
            int64_t lo = 0, hi = n;
            while (lo < hi) {
                int64_t mid = lo + ((hi - lo) >> 1);
                if (rowptr[mid] < e)
                    lo = mid + 1;
                else
                    hi = mid;
            }
            if (rowptr[lo] != e)
                bad |= 4;
        }
    }
    if (bad)
        atomicOr(flag, bad);
}

void launch_csr_check(const Launch &L, const int64_t *rowptr, const int32_t *col, int64_t n, int64_t nnz, int32_t *flag,
                      unsigned long long *maxdeg)
{
    hipLaunchKernelGGL(csr_check_rows_kernel, dim3(grid_for(L, (n + 255) / 256, 16)), dim3(256), 0, L.stream, rowptr,
                       n, nnz, flag, maxdeg);
    if (nnz > 0)
        hipLaunchKernelGGL(csr_check_cols_kernel, dim3(grid_for(L, (nnz + 255) / 256, 16)), dim3(256), 0, L.stream,
                           rowptr, col, n, nnz, flag);
}

// ---------------------------------------------------------------------------------------------
// Seed verification: Q^L has one nonzero per batch vertex (Sec. 4.1.1 / 4.2.1), so an id must be
// in range and must not repeat inside its minibatch.  Uses (and afterwards restores) the
// minibatch's vertex set.  flag bit 0: out of range, bit 1: repeated.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void validate_seeds_kernel(const int32_t *__restrict__ seeds, int64_t total, int32_t b,
                                                             int64_t n, VSet vs, int32_t *flag)
{
    for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = seeds[x];
        if (v < 0 || (int64_t)v >= n) {
            atomicOr(flag, 1);
            continue;
        }
        const int64_t i = x / b;
        const uint32_t bit = 1u << (v & 31);
        const uint32_t old = atomicOr(&vs.words[i * vs.nw + (v >> 5)], bit);
        if (old & bit)
            atomicOr(flag, 2);
    }
}

__global__ __launch_bounds__(256) void clear_seed_bits_kernel(const int32_t *__restrict__ seeds, int64_t total, int32_t b,
                                                              int64_t n, VSet vs)
{
    for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = seeds[x];
        if (v < 0 || (int64_t)v >= n)
            continue;
        vs.words[(x / b) * vs.nw + (v >> 5)] = 0u;
    }
}

void launch_validate_seeds(const Launch &L, const int32_t *seeds, int32_t k, int32_t b, int64_t n, const VSet &vs,
                           int32_t *flag)
{
    const int64_t total = (int64_t)k * b;
    hipLaunchKernelGGL(validate_seeds_kernel, dim3(grid_for(L, (total + 255) / 256, 8)), dim3(256), 0, L.stream, seeds,
                       total, b, n, vs, flag);
}

void launch_clear_seed_bits(const Launch &L, const int32_t *seeds, int32_t k, int32_t b, int64_t n, const VSet &vs)
{
    const int64_t total = (int64_t)k * b;
    hipLaunchKernelGGL(clear_seed_bits_kernel, dim3(grid_for(L, (total + 255) / 256, 8)), dim3(256), 0, L.stream, seeds,
                       total, b, n, vs);
}

__global__ void iota_offsets_kernel(int64_t *off, int32_t k, int64_t step)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i <= k; i += (int64_t)gridDim.x * blockDim.x)
        off[i] = i * step;
}

void launch_iota_offsets(const Launch &L, int64_t *off, int32_t k, int64_t step)
{
    hipLaunchKernelGGL(iota_offsets_kernel, dim3(grid_for(L, ((int64_t)k + 256) / 256, 4)), dim3(256), 0, L.stream, off,
                       k, step);
}

// ---------------------------------------------------------------------------------------------
// Tiles never straddle two minibatches: segment i (rows, or entries of P) is cut into
// ceil(len_i / tile) tiles; seg_tileoff is the exclusive scan of those counts (k+1 entries).
// Single workgroup: k is small (the number of minibatches).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void plan_tiles_kernel(const int64_t *__restrict__ seg_off, int32_t k, int32_t tile,
                                                          int64_t *seg_tileoff, unsigned long long *max_out)
{
    __shared__ int64_t smem[16];
    __shared__ int64_t carry_s;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (int32_t base = 0; base < k; base += 1024) {
        const int32_t i = base + threadIdx.x;
        int64_t cnt = 0;
        if (i < k)
            cnt = (seg_off[i + 1] - seg_off[i] + tile - 1) / tile;
        if (max_out && cnt > 0)
            atomicMax(max_out, (unsigned long long)cnt); // *max_out zeroed by the caller
        int64_t total;
        const int64_t ex = block_exclusive_scan<int64_t, 1024>(cnt, smem, total);
        const int64_t carry = carry_s;
        if (i < k)
            seg_tileoff[i] = carry + ex;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0)
        seg_tileoff[k] = carry_s;
}

void launch_plan_tiles(const Launch &L, const int64_t *seg_off, int32_t k, int32_t tile, int64_t *seg_tileoff,
                       int64_t *max_out)
{
    if (max_out)
        (void)hipMemsetAsync(max_out, 0, sizeof(int64_t), L.stream);
    hipLaunchKernelGGL(plan_tiles_kernel, dim3(1), dim3(1024), 0, L.stream, seg_off, k, tile, seg_tileoff,
                       reinterpret_cast<unsigned long long *>(max_out));
}

// three tilings of the same segments in one launch (one workgroup each)
__global__ __launch_bounds__(1024) void plan_tiles3_kernel(const int64_t *__restrict__ seg_off, int32_t k, int32_t tile0,
                                                           int64_t *off0, int32_t tile1, int64_t *off1, int32_t tile2,
                                                           int64_t *off2)
{
    __shared__ int64_t smem[16];
    __shared__ int64_t carry_s;
    const int32_t tile = blockIdx.x == 0 ? tile0 : blockIdx.x == 1 ? tile1 : tile2;
    int64_t *seg_tileoff = blockIdx.x == 0 ? off0 : blockIdx.x == 1 ? off1 : off2;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (int32_t base = 0; base < k; base += 1024) {
        const int32_t i = base + threadIdx.x;
        int64_t cnt = 0;
        if (i < k)
            cnt = (seg_off[i + 1] - seg_off[i] + tile - 1) / tile;
        int64_t total;
        const int64_t ex = block_exclusive_scan<int64_t, 1024>(cnt, smem, total);
        const int64_t carry = carry_s;
        if (i < k)
            seg_tileoff[i] = carry + ex;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0)
        seg_tileoff[k] = carry_s;
}

void launch_plan_tiles3(const Launch &L, const int64_t *seg_off, int32_t k, int32_t tile0, int64_t *off0, int32_t tile1,
                        int64_t *off1, int32_t tile2, int64_t *off2)
{
    hipLaunchKernelGGL(plan_tiles3_kernel, dim3(3), dim3(1024), 0, L.stream, seg_off, k, tile0, off0, tile1, off1, tile2,
                       off2);
}

// ---------------------------------------------------------------------------------------------
// In-place exclusive scan of an int64 array whose length lives on the device.  One workgroup,
// The arrays scanned here are per-tile sums and per-row counts (up to a few hundred thousand).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void scan_i64_kernel(int64_t *vals, const int64_t *__restrict__ count,
                                                        int64_t *total_out, int64_t *tail_ptr,
                                                        const int64_t *__restrict__ tail_idx)
{
    __shared__ int64_t smem[16];
    __shared__ int64_t carry_s;
    const int64_t m = *count;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    // 4 values per lane per step; the next step's values are on their way while this step is scanned
    int64_t nxt[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
        nxt[q] = ((int64_t)threadIdx.x * 4 + q < m) ? vals[(int64_t)threadIdx.x * 4 + q] : 0;
    for (int64_t base = 0; base < m; base += 4096) {
        const int64_t i0 = base + (int64_t)threadIdx.x * 4;
        int64_t v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v[q] = nxt[q];
            nxt[q] = (i0 + 4096 + q < m) ? vals[i0 + 4096 + q] : 0;
        }
        const int64_t mine = v[0] + v[1] + v[2] + v[3];
        int64_t total;
        int64_t ex = block_exclusive_scan<int64_t, 1024>(mine, smem, total) + carry_s;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i0 + q < m)
                vals[i0 + q] = ex;
            ex += v[q];
        }
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        vals[m] = carry_s;
        if (total_out)
            *total_out = carry_s;
        if (tail_ptr)
            tail_ptr[*tail_idx] = carry_s;
    }
}

// Long arrays, three steps: every workgroup scans its 4096 values in place and leaves their sum; one workgroup
// scans the sums; every workgroup adds what lies before it.
__global__ __launch_bounds__(1024) void scan_i64_chunks_kernel(int64_t *vals, const int64_t *__restrict__ count,
                                                               int64_t *__restrict__ sums)
{
    __shared__ int64_t smem[16];
    const int64_t m = *count;
    const int64_t nchunks = (m + 4095) / 4096;
    for (int64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const int64_t i0 = c * 4096 + (int64_t)threadIdx.x * 4;
        int64_t v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
            v[q] = (i0 + q < m) ? vals[i0 + q] : 0;
        int64_t total;
        int64_t ex = block_exclusive_scan<int64_t, 1024>(v[0] + v[1] + v[2] + v[3], smem, total);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (i0 + q < m)
                vals[i0 + q] = ex;
            ex += v[q];
        }
        if (threadIdx.x == 0)
            sums[c] = total;
        __syncthreads();
    }
    if (blockIdx.x == 0 && threadIdx.x == 0)
        sums[nchunks] = 0; // scanned along: becomes the grand total
}

__global__ __launch_bounds__(1024) void scan_i64_add_kernel(int64_t *vals, const int64_t *__restrict__ count,
                                                            const int64_t *__restrict__ sums, int64_t *total_out,
                                                            int64_t *tail_ptr, const int64_t *__restrict__ tail_idx)
{
    const int64_t m = *count;
    const int64_t nchunks = (m + 4095) / 4096;
    for (int64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const int64_t before = sums[c];
        const int64_t i0 = c * 4096 + (int64_t)threadIdx.x * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (i0 + q < m)
                vals[i0 + q] += before;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const int64_t total = sums[nchunks];
        vals[m] = total;
        if (total_out)
            *total_out = total;
        if (tail_ptr)
            tail_ptr[*tail_idx] = total;
    }
}

// Arrays of middling length, two steps: after the chunks kernel every workgroup adds up the sums of the chunks
// before its own by itself (at most kScanSelfChunks of them), so no workgroup scans the sums in between.
constexpr int64_t kScanSelfChunks = 1024;
__global__ __launch_bounds__(1024) void scan_i64_add_self_kernel(int64_t *vals, const int64_t *__restrict__ count,
                                                                 const int64_t *__restrict__ sums, int64_t *total_out,
                                                                 int64_t *tail_ptr, const int64_t *__restrict__ tail_idx)
{
    __shared__ int64_t smem[16];
    const int64_t m = *count;
    const int64_t nchunks = (m + 4095) / 4096; // <= kScanSelfChunks = the workgroup's size
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    for (int64_t c = blockIdx.x; c < nchunks + 1; c += gridDim.x) { // "chunk" nchunks: the grand total
        int64_t before = (int64_t)threadIdx.x < c ? sums[threadIdx.x] : 0;
        before = wave_sum(before);
        __syncthreads();
        if (lane == 0)
            smem[wave] = before;
        __syncthreads();
        before = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w)
            before += smem[w];
        if (c == nchunks) {
            if (threadIdx.x == 0) {
                vals[m] = before;
                if (total_out)
                    *total_out = before;
                if (tail_ptr)
                    tail_ptr[*tail_idx] = before;
            }
            continue;
        }
        const int64_t i0 = c * 4096 + (int64_t)threadIdx.x * 4;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (i0 + q < m)
                vals[i0 + q] += before;
    }
}

__global__ void scan_i64_count_kernel(const int64_t *__restrict__ count, int64_t *nchunks_plus_one)
{
    if (threadIdx.x == 0 && blockIdx.x == 0)
        *nchunks_plus_one = (*count + 4095) / 4096 + 1;
}

void launch_scan_i64(const Launch &L, int64_t *vals, const int64_t *count, int64_t *total_out, int64_t *tail_ptr,
                     const int64_t *tail_idx, int64_t count_bound)
{
    const int64_t chunks_bound = (count_bound + 4095) / 4096;
    if (count_bound > 32768 && chunks_bound <= kScanSelfChunks && L.scan_tmp && chunks_bound + 3 <= L.scan_tmp_len) {
        int64_t *sums = L.scan_tmp;
        hipLaunchKernelGGL(scan_i64_chunks_kernel, dim3(grid_for(L, chunks_bound, 2)), dim3(1024), 0, L.stream, vals, count, sums);
        hipLaunchKernelGGL(scan_i64_add_self_kernel, dim3(grid_for(L, chunks_bound + 1, 2)), dim3(1024), 0, L.stream, vals,
                           count, sums, total_out, tail_ptr, tail_idx);
        return;
    }
    if (count_bound > 32768 && L.scan_tmp && chunks_bound + 3 <= L.scan_tmp_len) { // one workgroup below that: fewer launches
        int64_t *sums = L.scan_tmp;                 // chunks_bound + 1 values
        int64_t *nsums = L.scan_tmp + chunks_bound + 2; // device-side length of `sums` for the middle scan
        const int grid = grid_for(L, chunks_bound, 2);
        hipLaunchKernelGGL(scan_i64_chunks_kernel, dim3(grid), dim3(1024), 0, L.stream, vals, count, sums);
        hipLaunchKernelGGL(scan_i64_count_kernel, dim3(1), dim3(64), 0, L.stream, count, nsums);
        // scans sums[0 .. nchunks] (the extra trailing zero turns into the grand total) and writes one value past it
        hipLaunchKernelGGL(scan_i64_kernel, dim3(1), dim3(1024), 0, L.stream, sums, nsums, nullptr, nullptr, nullptr);
        hipLaunchKernelGGL(scan_i64_add_kernel, dim3(grid), dim3(1024), 0, L.stream, vals, count, sums, total_out, tail_ptr,
                           tail_idx);
        return;
    }
    hipLaunchKernelGGL(scan_i64_kernel, dim3(1), dim3(1024), 0, L.stream, vals, count, total_out, tail_ptr, tail_idx);
}

// ---------------------------------------------------------------------------------------------
// Vertex set ranking.  After the bits of every sampled vertex are set:
//   count : set bits per chunk of 256 lines
//   scan  : per minibatch, exclusive scan over its chunks; per-minibatch totals -> mb_coloff
//   fill  : rank of every line's first vertex; the set vertices written out in ascending order
//           (the kept columns of EXTRACT = the next frontier)
// ---------------------------------------------------------------------------------------------
__device__ inline int line_popcount(const uint32_t *__restrict__ line_words, uint4 w[4])
{
    const uint4 *p = reinterpret_cast<const uint4 *>(line_words);
    int c = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        w[q] = p[q];
        c += __popc(w[q].x) + __popc(w[q].y) + __popc(w[q].z) + __popc(w[q].w);
    }
    return c;
}

__global__ __launch_bounds__(256) void vset_count_kernel(VSet vs, int32_t k)
{
    __shared__ int32_t wsum[4];
    const int64_t nblocks = (int64_t)k * vs.nc;
    for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int64_t i = blk / vs.nc;
        const int64_t line = (blk % vs.nc) * kChunkLines + threadIdx.x;
        int cnt = 0;
        if (line < vs.nl) {
            uint4 w[4];
            cnt = line_popcount(vs.words + i * vs.nw + line * kLineWords, w);
        }
        cnt = wave_sum(cnt);
        __syncthreads();
        if ((threadIdx.x & (kWave - 1)) == 0)
            wsum[threadIdx.x / kWave] = cnt;
        __syncthreads();
        if (threadIdx.x == 0)
            vs.chunk_off[blk] = (int64_t)wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
}

// one workgroup per minibatch: exclusive scan of its nc chunk counts in place; mb_count[i] = total
__global__ __launch_bounds__(1024) void chunk_scan_kernel(int64_t *chunk_off, int32_t nc, int64_t *mb_count)
{
    __shared__ int64_t smem[16];
    __shared__ int64_t carry_s;
    int64_t *c = chunk_off + (int64_t)blockIdx.x * nc;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (int32_t base = 0; base < nc; base += 1024) {
        const int32_t q = base + threadIdx.x;
        const int64_t v = q < nc ? c[q] : 0;
        int64_t total;
        const int64_t ex = block_exclusive_scan<int64_t, 1024>(v, smem, total);
        const int64_t carry = carry_s;
        if (q < nc)
            c[q] = carry + ex;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0)
        mb_count[blockIdx.x] = carry_s;
}

// mb_coloff = exclusive scan of mb_count over the k minibatches (k+1 entries); *ncols_out = total
__global__ __launch_bounds__(1024) void offsets_from_counts_kernel(const int64_t *__restrict__ mb_count, int32_t k,
                                                                   int64_t *mb_off, int64_t *total_out)
{
    __shared__ int64_t smem[16];
    __shared__ int64_t carry_s;
    if (threadIdx.x == 0)
        carry_s = 0;
    __syncthreads();
    for (int32_t base = 0; base < k; base += 1024) {
        const int32_t i = base + threadIdx.x;
        const int64_t v = i < k ? mb_count[i] : 0;
        int64_t total;
        const int64_t ex = block_exclusive_scan<int64_t, 1024>(v, smem, total);
        const int64_t carry = carry_s;
        if (i < k)
            mb_off[i] = carry + ex;
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        mb_off[k] = carry_s;
        if (total_out)
            *total_out = carry_s;
    }
}

__global__ __launch_bounds__(256) void vset_fill_kernel(VSet vs, int32_t k, const int64_t *__restrict__ mb_coloff,
                                                        int32_t *__restrict__ col_vertex)
{
    __shared__ int32_t smem[4];
    const int64_t nblocks = (int64_t)k * vs.nc;
    for (int64_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
        const int64_t i = blk / vs.nc;
        const int64_t line = (blk % vs.nc) * kChunkLines + threadIdx.x;
        uint4 w[4];
        int cnt = 0;
        if (line < vs.nl)
            cnt = line_popcount(vs.words + i * vs.nw + line * kLineWords, w);
        int total;
        const int ex = block_exclusive_scan<int32_t, 256>(cnt, smem, total);
        if (line < vs.nl) {
            const int64_t rank0 = vs.chunk_off[blk] + ex; // < 2^31: at most n distinct vertices per minibatch
            vs.line_prefix[i * vs.nl + line] = (uint32_t)rank0;
            if (cnt) {
                int32_t *dst = col_vertex + mb_coloff[i] + rank0;
                const uint32_t ww[16] = {w[0].x, w[0].y, w[0].z, w[0].w, w[1].x, w[1].y, w[1].z, w[1].w,
                                         w[2].x, w[2].y, w[2].z, w[2].w, w[3].x, w[3].y, w[3].z, w[3].w};
                const int32_t id0 = (int32_t)(line * kLineBits);
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    uint32_t x = ww[q];
                    while (x) {
                        const int bit = __ffs(x) - 1;
                        x &= x - 1;
                        *dst++ = id0 + q * 32 + bit;
                    }
                }
            }
        }
    }
}

void launch_offsets_from_counts(const Launch &L, const int64_t *mb_count, int32_t k, int64_t *mb_off, int64_t *total_out)
{
    hipLaunchKernelGGL(offsets_from_counts_kernel, dim3(1), dim3(1024), 0, L.stream, mb_count, k, mb_off, total_out);
}

// Seed verification without a vertex set: one workgroup sorts a minibatch's b seeds in LDS
// (bitonic network over the next power of two, padded with distinct values above every id) and
// looks for equal neighbours.  flag bit 0: out of range, bit 1: repeated.
__global__ __launch_bounds__(1024) void validate_seeds_sorted_kernel(const int32_t *__restrict__ seeds, int32_t k,
                                                                     int32_t b, int32_t m /*pow2 >= b*/, int64_t n,
                                                                     int32_t *flag)
{
    __shared__ uint32_t key[kMaxSortedSeeds];
    for (int32_t i = blockIdx.x; i < k; i += gridDim.x) {
        int bad = 0;
        for (int32_t j = threadIdx.x; j < m; j += 1024) {
            uint32_t v = 0x80000000u + (uint32_t)j; // padding: distinct, above every valid id
            if (j < b) {
                const int32_t sv = seeds[(int64_t)i * b + j];
                if (sv < 0 || (int64_t)sv >= n)
                    bad |= 1; // keeps its padding value so that it cannot fake a repeat
                else
                    v = (uint32_t)sv;
            }
            key[j] = v;
        }
        __syncthreads();
        for (int32_t size = 2; size <= m; size <<= 1) {
            for (int32_t stride = size >> 1; stride > 0; stride >>= 1) {
                for (int32_t j = threadIdx.x; j < m; j += 1024) {
                    const int32_t partner = j ^ stride;
                    if (partner > j) {
                        const bool up = (j & size) == 0;
                        const uint32_t x = key[j], y = key[partner];
                        if ((x > y) == up) {
                            key[j] = y;
                            key[partner] = x;
                        }
                    }
                }
                __syncthreads();
            }
        }
        for (int32_t j = threadIdx.x; j + 1 < m; j += 1024)
            if (key[j] == key[j + 1])
                bad |= 2;
        if (bad)
            atomicOr(flag, bad);
        __syncthreads();
    }
}

void launch_validate_seeds_sorted(const Launch &L, const int32_t *seeds, int32_t k, int32_t b, int64_t n, int32_t *flag)
{
    int32_t m = 2;
    while (m < b)
        m <<= 1;
    hipLaunchKernelGGL(validate_seeds_sorted_kernel, dim3(grid_for(L, k, 2)), dim3(1024), 0, L.stream, seeds, k, b, m, n,
                       flag);
}

void launch_chunk_scan(const Launch &L, int64_t *chunk_off, int32_t k, int32_t nc, int64_t *mb_off, int64_t *total_out)
{
    // per-minibatch totals are parked in the k entries after the k*nc chunk entries of chunk_off
    int64_t *mb_count = chunk_off + (int64_t)k * nc;
    hipLaunchKernelGGL(chunk_scan_kernel, dim3(k), dim3(1024), 0, L.stream, chunk_off, nc, mb_count);
    hipLaunchKernelGGL(offsets_from_counts_kernel, dim3(1), dim3(1024), 0, L.stream, mb_count, k, mb_off, total_out);
}

void launch_vset_rank(const Launch &L, const VSet &vs, int32_t k, int64_t *mb_coloff, int32_t *col_vertex,
                      int64_t *ncols_out)
{
    const int64_t nblocks = (int64_t)k * vs.nc;
    hipLaunchKernelGGL(vset_count_kernel, dim3(grid_for(L, nblocks, 16)), dim3(256), 0, L.stream, vs, k);
    launch_chunk_scan(L, vs.chunk_off, k, vs.nc, mb_coloff, ncols_out);
    hipLaunchKernelGGL(vset_fill_kernel, dim3(grid_for(L, nblocks, 16)), dim3(256), 0, L.stream, vs, k, mb_coloff,
                       col_vertex);
}

// Restore the all-zero invariant: every set bit belongs to a vertex listed in col_vertex.
__global__ __launch_bounds__(256) void vset_clear_kernel(VSet vs, int32_t k, const int64_t *__restrict__ mb_coloff,
                                                         const int32_t *__restrict__ col_vertex)
{
    const int64_t total = mb_coloff[k];
    for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (int64_t)gridDim.x * blockDim.x) {
        const int i = locate_segment(mb_coloff, k, x);
        const int32_t v = col_vertex[x];
        vs.words[(int64_t)i * vs.nw + (v >> 5)] = 0u;
    }
}

void launch_vset_clear(const Launch &L, const VSet &vs, int32_t k, const int64_t *mb_coloff, const int32_t *col_vertex,
                       int64_t ncols_bound)
{
    hipLaunchKernelGGL(vset_clear_kernel, dim3(grid_for(L, (ncols_bound + 255) / 256, 8)), dim3(256), 0, L.stream, vs,
                       k, mb_coloff, col_vertex);
}

} // namespace bms
