// Rate probes for one MI355X: what the chip does on the two access patterns that bound the sampling kernels.
// Measurement aids for bench.py (--line-probe, --lds-probe); no part of libbms.so and of no use to a caller of it.
//
//   random rows   every lane reads the first `entries` 4-byte entries of a row that starts at a random 4-byte
//                 aligned place of a large array: the pattern of P = Q A with one nonzero per row of Q (Sec. 4.1.1)
//                 when the rows are short.  The rate in 128-byte lines per second is the ceiling of the node-wise
//                 row and sampling kernels.
//   LDS adds      16 waves of one workgroup per compute unit add into 128 KB of LDS at random places: the pattern
//                 of the layer-wise count accumulation (Sec. 4.2.1).  The time per wave instruction bounds the
//                 instructions a compute unit can spend per neighbour.
#include <hip/hip_runtime.h>
#include <cstdint>

namespace {

template <int ENTRIES>
__global__ __launch_bounds__(256) void random_rows_kernel(const int32_t *__restrict__ array,
                                                          const int64_t *__restrict__ start, int64_t nrows,
                                                          int32_t *sink)
{
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x, gsz = (int64_t)gridDim.x * 256;
    int32_t acc = 0;
    for (int64_t r = gid; r < nrows; r += gsz) {
        const int32_t *src = array + start[r];
        int32_t v[ENTRIES];
#pragma unroll
        for (int j = 0; j < ENTRIES; ++j)
            v[j] = src[j];
#pragma unroll
        for (int j = 0; j < ENTRIES; ++j)
            acc += v[j];
    }
    if (acc == 0x12345678) // never with the zero-filled array of the probe: keeps the loads alive
        *sink = acc;
}

constexpr int kLdsWords = 32768; // 128 KB
template <int MODE>
__global__ __launch_bounds__(1024) void lds_ops_kernel(uint32_t *ticks, int iters, uint32_t active_every)
{
    extern __shared__ uint32_t lds[];
    const int tid = threadIdx.x;
    for (int x = tid; x < kLdsWords; x += 1024)
        lds[x] = 0;
    __syncthreads();
    uint32_t s = tid * 2654435761u + blockIdx.x * 97u + 12345u;
    const bool on = (tid % active_every) == 0;
    const uint64_t t0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            s = s * 1664525u + 1013904223u;
            const uint32_t x = s >> 16; // a 16-bit counter index
            if (on) {
                if (MODE == 0)
                    atomicAdd(&lds[x >> 1], 1u << ((x & 1u) * 16));
                else
                    lds[x >> 1] = s;
            }
        }
    }
    __syncthreads();
    const uint64_t t1 = wall_clock64();
    uint32_t acc = 0;
    for (int x = tid; x < kLdsWords; x += 1024)
        acc += lds[x];
    if (tid == 0)
        ticks[blockIdx.x] = (uint32_t)(t1 - t0); // 100 MHz
    if (acc == 0xdeadbeefu && s == 1u)
        ticks[0] = acc;
}

} // namespace

extern "C" {

// Enqueues one pass over `nrows` rows on `stream`; array (n_array int32, device), start (nrows int64, device, every
// value in [0, n_array - entries]), sink (one int32, device).  entries is 1 or 8.  0 = ok, -1 = bad argument or launch.
int bms_probe_random_rows(const int32_t *array, int64_t n_array, const int64_t *start, int64_t nrows, int32_t entries,
                          int32_t workgroups, int32_t *sink, void *stream)
{
    if (!array || !start || !sink || n_array < 8 || nrows < 0 || workgroups < 1 || (entries != 1 && entries != 8))
        return -1;
    if (entries == 1)
        hipLaunchKernelGGL(random_rows_kernel<1>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, array, start, nrows, sink);
    else
        hipLaunchKernelGGL(random_rows_kernel<8>, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, array, start, nrows, sink);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

// One 1024-thread workgroup per entry of ticks (device, `workgroups` uint32), each doing iters x 16 LDS
// instructions per wave; mode 0 = 16-bit adds packed in 32-bit words at random places, 1 = 32-bit stores at random
// places; every `active_every`-th lane takes part.  ticks[w] = 100 MHz ticks workgroup w spent.  0 = ok.
int bms_probe_lds_ops(uint32_t *ticks, int32_t workgroups, int32_t iters, int32_t mode, int32_t active_every, void *stream)
{
    if (!ticks || workgroups < 1 || iters < 1 || active_every < 1 || mode < 0 || mode > 1)
        return -1;
    const void *fn = mode == 0 ? (const void *)lds_ops_kernel<0> : (const void *)lds_ops_kernel<1>;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsWords * 4) != hipSuccess)
        (void)hipGetLastError();
    if (mode == 0)
        hipLaunchKernelGGL(lds_ops_kernel<0>, dim3(workgroups), dim3(1024), kLdsWords * 4, (hipStream_t)stream, ticks, iters, (uint32_t)active_every);
    else
        hipLaunchKernelGGL(lds_ops_kernel<1>, dim3(workgroups), dim3(1024), kLdsWords * 4, (hipStream_t)stream, ticks, iters, (uint32_t)active_every);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

} // extern "C"
