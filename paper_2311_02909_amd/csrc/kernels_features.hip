// Feature fetching, the part one GPU does (Sec. 6.2 of arxiv 2311.02909): H_i = the rows of the
// feature matrix H of the vertices in the last frontier.  A pure row gather, bound by HBM bandwidth:
// every row is read once and written once (4 f bytes each way, f = 100..128 in the paper's datasets).
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

// 2^lanes_log2 lanes share a row and move VEC floats each per access; every lane has four rows in
// flight.  An id outside [0, n) gives a row of zeros and raises *flag.
template <int VEC>
__global__ __launch_bounds__(256) void feature_fetch_kernel(const float *__restrict__ H, int64_t n, int32_t f,
                                                            const int32_t *__restrict__ ids, int64_t m,
                                                            float *__restrict__ out, int32_t *flag, int lanes_log2)
{
    struct alignas(4 * VEC) Vec {
        float x[VEC];
    };
    const int per_row = f / VEC; // accesses per row
    const int lanes = 1 << lanes_log2;
    const int sub = threadIdx.x & (lanes - 1);
    const int64_t rows_per_block = 256 >> lanes_log2;
    const int64_t stride = (int64_t)gridDim.x * rows_per_block;
    for (int64_t j0 = (int64_t)blockIdx.x * rows_per_block + (threadIdx.x >> lanes_log2); j0 < m; j0 += 4 * stride) {
        int64_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t j = j0 + u * stride;
            v[u] = j < m ? (int64_t)ids[j] : 0;
        }
        for (int x = sub; x < per_row; x += lanes) {
            Vec val[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t j = j0 + u * stride;
                val[u] = Vec{};
                if (j < m && v[u] >= 0 && v[u] < n)
                    val[u] = reinterpret_cast<const Vec *>(H + v[u] * f)[x];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t j = j0 + u * stride;
                if (j < m)
                    reinterpret_cast<Vec *>(out + j * f)[x] = val[u];
            }
        }
        if (sub == 0) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (j0 + u * stride < m && (v[u] < 0 || v[u] >= n))
                    *flag = 1;
        }
    }
}

void launch_feature_fetch(const Launch &L, const float *H, int64_t n, int32_t f, const int32_t *ids, int64_t m,
                          float *out, int32_t *flag)
{
    if (m <= 0)
        return;
    const bool wide = f % 4 == 0 && (reinterpret_cast<uintptr_t>(H) & 15) == 0 && (reinterpret_cast<uintptr_t>(out) & 15) == 0;
    const int per_row = wide ? f / 4 : f;
    int lanes_log2 = 0;
    while ((1 << lanes_log2) < per_row && lanes_log2 < 6)
        ++lanes_log2;
    const int64_t rows_per_block = 256 >> lanes_log2;
    const int grid = grid_for(L, (m + 4 * rows_per_block - 1) / (4 * rows_per_block), 8);
    if (wide)
        hipLaunchKernelGGL(feature_fetch_kernel<4>, dim3(grid), dim3(256), 0, L.stream, H, n, f, ids, m, out, flag, lanes_log2);
    else
        hipLaunchKernelGGL(feature_fetch_kernel<1>, dim3(grid), dim3(256), 0, L.stream, H, n, f, ids, m, out, flag, lanes_log2);
}

} // namespace bms

namespace bms {

// Forward neighbourhood aggregation of one hop (Sec. 6.2): the SpMM between the stacked sampled adjacency
// (all entries 1) and the feature rows of its columns.  2^lanes_log2 lanes share an output row and hold
// VEC features each per access; the row's entries are added in ascending order in fp32, four gathered
// rows in flight.  mean != 0 divides by the number of entries (rows without entries give zeros).
template <int VEC>
__global__ __launch_bounds__(256) void aggregate_kernel(AggArgs a, int lanes_log2)
{
    struct alignas(4 * VEC) Vec {
        float x[VEC];
    };
    const int per_row = a.f / VEC;
    const int lanes = 1 << lanes_log2;
    const int sub = threadIdx.x & (lanes - 1);
    const int64_t rows_per_block = 256 >> lanes_log2;
    for (int64_t r = (int64_t)blockIdx.x * rows_per_block + (threadIdx.x >> lanes_log2); r < a.rows;
         r += (int64_t)gridDim.x * rows_per_block) {
        const int64_t e0 = a.rowptr[r], e1 = a.rowptr[r + 1];
        const int64_t c0 = a.mb_coloff[locate_segment(a.mb_rowoff, a.k, r)];
        const float len = (float)(e1 - e0);
        for (int x = sub; x < per_row; x += lanes) {
            Vec acc = Vec{};
            for (int64_t e = e0; e < e1; e += 4) {
                Vec v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    v[u] = Vec{};
                    if (e + u < e1)
                        v[u] = reinterpret_cast<const Vec *>(a.X + (c0 + a.col[e + u]) * a.f)[x];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (e + u < e1) { // entry order
#pragma unroll
                        for (int q = 0; q < VEC; ++q)
                            acc.x[q] += v[u].x[q];
                    }
            }
            if (a.mean && e1 > e0) {
#pragma unroll
                for (int q = 0; q < VEC; ++q)
                    acc.x[q] = acc.x[q] / len;
            }
            reinterpret_cast<Vec *>(a.out + r * a.f)[x] = acc;
        }
    }
}

void launch_aggregate(const Launch &L, const AggArgs &a)
{
    if (a.rows <= 0)
        return;
    const bool wide = a.f % 4 == 0 && (reinterpret_cast<uintptr_t>(a.X) & 15) == 0 && (reinterpret_cast<uintptr_t>(a.out) & 15) == 0;
    const int per_row = wide ? a.f / 4 : a.f;
    int lanes_log2 = 0;
    while ((1 << lanes_log2) < per_row && lanes_log2 < 6)
        ++lanes_log2;
    const int64_t rows_per_block = 256 >> lanes_log2;
    const int grid = grid_for(L, (a.rows + rows_per_block - 1) / rows_per_block, 8);
    if (wide)
        hipLaunchKernelGGL(aggregate_kernel<4>, dim3(grid), dim3(256), 0, L.stream, a, lanes_log2);
    else
        hipLaunchKernelGGL(aggregate_kernel<1>, dim3(grid), dim3(256), 0, L.stream, a, lanes_log2);
}

} // namespace bms
