// EXTRACT for the node-wise sampler on large vertex ranges (Sec. 4.1.3: "remove empty columns"):
// one workgroup per minibatch turns the minibatch's sampled global ids into local column indices
// and the ascending list of distinct ids, without any per-minibatch structure of size n in HBM.
//
//   A  partition the minibatch's (id, position) pairs by id range into buckets of 2^18 ids
//      (LDS histogram, LDS scan, one scattered 8-byte store per sampled edge);
//   B  per bucket, a 2^18-bit bitmap held in LDS: set the bits, popcount-scan the words, emit the
//      set ids in ascending order, and give every pair its rank = distinct ids before it.
//
// Buckets are visited in ascending id order and the bitmap orders ids inside a bucket, so the
// result is the ascending order whatever order the pairs landed in (the partition need not be
// stable).  All synchronisation is workgroup-local.
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

constexpr int kBucketWords = 1 << (kBucketBits - 5); // 8192 words = 32 KB

// mb_edgeoff[i] = first entry of minibatch i in the stacked column array
__global__ void mb_edge_offsets_kernel(const int64_t *__restrict__ out_rowptr, const int64_t *__restrict__ mb_rowoff,
                                       int32_t k, int64_t *mb_edgeoff)
{
    for (int32_t i = blockIdx.x * blockDim.x + threadIdx.x; i <= k; i += gridDim.x * blockDim.x)
        mb_edgeoff[i] = out_rowptr[mb_rowoff[i]];
}

__global__ __launch_bounds__(1024) void nw_dedup_bucket_kernel(DedupArgs a)
{
    __shared__ uint32_t bm[kBucketWords];      // bitmap of the current bucket
    __shared__ uint32_t pre[kBucketWords / 2]; // set bits before each pair of words
    __shared__ uint32_t cur[kMaxBuckets];      // bucket counts -> starts -> ends
    __shared__ uint32_t smem[16];
    __shared__ uint32_t carry_s;
    const int tid = threadIdx.x;
    const int32_t nb = a.nbuckets;
    for (int32_t i = blockIdx.x; i < a.k; i += gridDim.x) {
        const int64_t e0 = a.mb_edgeoff[i];
        const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
        int32_t *__restrict__ col = a.col + e0;        // in: global ids, out: local column indices
        uint64_t *__restrict__ pairs = a.pairs + e0;
        int32_t *__restrict__ uniq = a.uniq + e0;

        // ---- A: partition by id range ----
        for (int32_t b = tid; b < nb; b += 1024)
            cur[b] = 0;
        if (tid == 0)
            carry_s = 0;
        __syncthreads();
        for (uint32_t j = tid; j < N; j += 1024)
            atomicAdd(&cur[(uint32_t)col[j] >> kBucketBits], 1u);
        __syncthreads();
        for (int32_t base = 0; base < nb; base += 1024) {
            const int32_t b = base + tid;
            const uint32_t v = b < nb ? cur[b] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<uint32_t, 1024>(v, smem, total);
            const uint32_t carry = carry_s;
            if (b < nb)
                cur[b] = carry + ex;
            __syncthreads();
            if (tid == 0)
                carry_s = carry + total;
            __syncthreads();
        }
        for (uint32_t j = tid; j < N; j += 1024) {
            const uint32_t g = (uint32_t)col[j];
            const uint32_t pos = atomicAdd(&cur[g >> kBucketBits], 1u);
            pairs[pos] = ((uint64_t)g << 32) | (uint64_t)j;
        }
        __syncthreads(); // cur[b] is now the end of bucket b; its start is cur[b-1]

        // ---- B: per bucket, bitmap in LDS ----
        uint32_t ubase = 0; // distinct ids in the buckets before this one (same value in every lane)
        for (int32_t b = 0; b < nb; ++b) {
            const uint32_t s = b ? cur[b - 1] : 0u;
            const uint32_t e = cur[b];
            if (s == e)
                continue;
            uint4 *bm4 = reinterpret_cast<uint4 *>(bm);
            bm4[2 * tid] = make_uint4(0, 0, 0, 0);
            bm4[2 * tid + 1] = make_uint4(0, 0, 0, 0);
            __syncthreads();
            for (uint32_t j = s + tid; j < e; j += 1024) {
                const uint32_t l = (uint32_t)(pairs[j] >> 32) & ((1u << kBucketBits) - 1u);
                atomicOr(&bm[l >> 5], 1u << (l & 31));
            }
            __syncthreads();
            // lane t owns words [8t, 8t+8)
            const uint4 w0 = bm4[2 * tid], w1 = bm4[2 * tid + 1];
            const uint32_t w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
            uint32_t mine = 0;
#pragma unroll
            for (int q = 0; q < 8; ++q)
                mine += __popc(w[q]);
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<uint32_t, 1024>(mine, smem, total);
            uint32_t run = ex;
#pragma unroll
            for (int q = 0; q < 8; q += 2) {
                pre[4 * tid + (q >> 1)] = run;
                run += __popc(w[q]) + __popc(w[q + 1]);
            }
            if (mine) {
                int32_t *dst = uniq + ubase + ex;
                const uint32_t id0 = ((uint32_t)b << kBucketBits) + (uint32_t)tid * 256u;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    uint32_t x = w[q];
                    while (x) {
                        const int bit = __ffs(x) - 1;
                        x &= x - 1;
                        *dst++ = (int32_t)(id0 + q * 32 + bit);
                    }
                }
            }
            __syncthreads();
            for (uint32_t j = s + tid; j < e; j += 1024) {
                const uint64_t p = pairs[j];
                const uint32_t l = (uint32_t)(p >> 32) & ((1u << kBucketBits) - 1u);
                const uint32_t wi = l >> 5;
                uint32_t r = ubase + pre[wi >> 1] + __popc(bm[wi] & ((1u << (l & 31)) - 1u));
                if (wi & 1)
                    r += __popc(bm[wi - 1]);
                col[(uint32_t)p] = (int32_t)r;
            }
            ubase += total;
            __syncthreads();
        }
        if (tid == 0)
            a.mb_count[i] = ubase;
    }
}

// col_vertex[mb_coloff[i] + c] = uniq[mb_edgeoff[i] + c]
__global__ __launch_bounds__(256) void compact_unique_kernel(DedupArgs a, const int64_t *__restrict__ mb_coloff,
                                                             int32_t *__restrict__ col_vertex)
{
    const int64_t total = mb_coloff[a.k];
    for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < total; x += (int64_t)gridDim.x * blockDim.x) {
        const int i = locate_segment(mb_coloff, a.k, x);
        col_vertex[x] = a.uniq[a.mb_edgeoff[i] + (x - mb_coloff[i])];
    }
}

void launch_nw_dedup_bucket(const Launch &L, const DedupArgs &a, const int64_t *out_rowptr, const int64_t *mb_rowoff,
                            int64_t *mb_coloff, int32_t *col_vertex, int64_t *ncols_out, int64_t ncols_bound)
{
    hipLaunchKernelGGL(mb_edge_offsets_kernel, dim3((a.k + 256) / 256), dim3(256), 0, L.stream, out_rowptr, mb_rowoff,
                       a.k, a.mb_edgeoff);
    hipLaunchKernelGGL(nw_dedup_bucket_kernel, dim3(a.k), dim3(1024), 0, L.stream, a);
    launch_offsets_from_counts(L, a.mb_count, a.k, mb_coloff, ncols_out);
    hipLaunchKernelGGL(compact_unique_kernel, dim3(grid_for(L, (ncols_bound + 255) / 256, 8)), dim3(256), 0, L.stream,
                       a, mb_coloff, col_vertex);
}

} // namespace bms
