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
