// Device-side building blocks shared by the sampler kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bms {

constexpr int kWave = 64;
constexpr int kRowTile = 256;      // stacked rows handled by one workgroup iteration (one row per lane)
constexpr int kLineWords = 16;     // a vertex-set "line": 16 x 32-bit words = 512 vertex ids = 64 bytes
constexpr int kLineBits = 512;
constexpr int kChunkLines = 256;   // lines ranked by one workgroup (131072 vertex ids)

// ---------------------------------------------------------------------------------------------
// Counter-based random stream: a stateless hash of (seed, hop, minibatch, vertex, draw index).
// 64-bit work happens once per distribution (the key); every draw is 32-bit arithmetic.
// ---------------------------------------------------------------------------------------------
__host__ __device__ inline uint64_t mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

__host__ __device__ inline uint32_t fin32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7FEB352DU;
    x ^= x >> 15;
    x *= 0x846CA68BU;
    x ^= x >> 16;
    return x;
}

// key of the (seed, hop) pair; computed on the host once per hop
__host__ __device__ inline uint64_t hop_key(uint64_t seed, int32_t hop)
{
    return mix64(seed ^ (0x9E3779B97F4A7C15ULL * (uint64_t)(hop + 1)));
}

__host__ __device__ inline uint64_t row_key(uint64_t hopkey, uint32_t mb, uint32_t vertex)
{
    return mix64(hopkey ^ (((uint64_t)mb << 32) | (uint64_t)vertex));
}

__device__ inline uint32_t draw32(uint64_t key, uint32_t j)
{
    return fin32(fin32((uint32_t)key + j * 0x9E3779B9U) ^ (uint32_t)(key >> 32));
}

__device__ inline uint64_t draw64(uint64_t key, uint32_t j)
{
    return ((uint64_t)draw32(key, 2u * j) << 32) | (uint64_t)draw32(key, 2u * j + 1u);
}

__device__ inline uint32_t bounded32(uint32_t x, uint32_t m) { return __umulhi(x, m); }
__device__ inline uint64_t bounded64(uint64_t x, uint64_t w) { return __umul64hi(x, w); }

constexpr uint32_t kNoVertex = 0xFFFFFFFFu;

// ---------------------------------------------------------------------------------------------
// Scans
// ---------------------------------------------------------------------------------------------
template <class T>
__device__ inline T wave_inclusive_scan(T v)
{
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T o = __shfl_up(v, d, kWave);
        if (lane >= d)
            v += o;
    }
    return v;
}

// The same for 32-bit counts through the vector unit's lane-permute paths only (no LDS crossbar): shifts inside
// each row of 16 lanes, then the last lane of rows 0 and 2 broadcast into rows 1 and 3, then lane 31 into rows 2, 3.
__device__ inline uint32_t wave_inclusive_scan_dpp(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111 /* row_shr:1 */, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112 /* row_shr:2 */, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114 /* row_shr:4 */, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118 /* row_shr:8 */, 0xF, 0xF, true);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142 /* row_bcast:15 */, 0xA, 0xF, false);
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143 /* row_bcast:31 */, 0xC, 0xF, false);
    return v;
}

template <class T>
__device__ inline T wave_sum(T v)
{
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1)
        v += __shfl_xor(v, d, kWave);
    return v;
}

// Exclusive scan over the NT threads of a workgroup.  `smem` holds NT/64 values of T.
// Contains two barriers; smem may be reused after the call returns on all threads
// only after another barrier (the callers loop with barriers in between).
template <class T, int NT>
__device__ inline T block_exclusive_scan(T v, T *smem, T &total)
{
    constexpr int NW = NT / kWave;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    T inc = wave_inclusive_scan(v);
    __syncthreads(); // protects smem against readers of a previous call
    if (lane == kWave - 1)
        smem[wave] = inc;
    __syncthreads();
    T before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        T x = smem[w];
        if (w < wave)
            before += x;
        all += x;
    }
    total = all;
    return before + inc - v;
}

// Largest i in [0,k) with off[i] <= t, given off[0] <= t < off[k] (off ascending, k >= 1).
__device__ inline int locate_segment(const int64_t *__restrict__ off, int k, int64_t t)
{
    int lo = 0, hi = k;
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (off[mid] <= t)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

// Rank of vertex g inside one minibatch's vertex set: set bits before it = line_prefix of its
// 64-byte line + set bits before it inside the line.  `words`/`line_prefix` point at the
// minibatch's own slice.
__device__ inline int32_t vset_rank_of(const uint32_t *__restrict__ words, const uint32_t *__restrict__ line_prefix,
                                       int32_t g)
{
    const int32_t line = g >> 9;
    const int32_t w = (g >> 5) & (kLineWords - 1);
    const uint4 *p = reinterpret_cast<const uint4 *>(words + (int64_t)line * kLineWords);
    uint32_t rank = line_prefix[line];
    const int nq = w >> 2; // whole 16-byte quarters before the word
    for (int q = 0; q < nq; ++q) {
        const uint4 x = p[q];
        rank += __popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w);
    }
    const uint4 x = p[nq];
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
    const int rem = w & 3;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (q < rem)
            rank += __popc(xs[q]);
        else if (q == rem)
            rank += __popc(xs[q] & ((1u << (g & 31)) - 1u));
    }
    return (int32_t)rank;
}

__device__ inline bool vset_test(const uint32_t *__restrict__ words, int32_t g)
{
    return (words[g >> 5] >> (g & 31)) & 1u;
}

} // namespace bms
