// EXTRACT for the node-wise sampler on large vertex ranges (Sec. 4.1.3: "remove empty columns"):
// one workgroup per minibatch turns the minibatch's sampled global ids into local column indices
// and the ascending list of distinct ids, without any per-minibatch structure of size n in HBM.
// Work is proportional to the number of sampled edges of the minibatch, not to n.
//
//   A  partition the minibatch's (id, position) pairs by id range into bins of 2^15 ids
//      (LDS histogram, LDS scan, one scattered 8-byte store per sampled edge);
//   B  every wave owns a contiguous run of bins (balanced by element count) and walks it in
//      groups: consecutive bins holding <= 64 pairs together are sorted in registers (one pair per
//      lane, 64-lane bitonic network on id-within-group << 6 | lane), a bin holding more than 64
//      pairs is ranked with a 2^15-bit bitmap in LDS.  Either way every pair learns its rank among
//      the distinct ids of its group, every distinct id is noted once, and the group's distinct
//      count is recorded;
//      a workgroup scan turns the counts into "distinct ids before the group";
//   C  (second kernel, all compute units) adds that base: local column = base + rank, and writes
//      the distinct ids to their final place in the next frontier.
//
// Bins are ascending id ranges, groups are runs of bins, and ids are ordered inside a group, so the
// result is the ascending order whatever order the pairs landed in (the partition need not be
// stable).  All synchronisation is workgroup-local; no wave ever waits on another except at
// workgroup barriers.
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

constexpr int kBinWords = 1 << (kBucketBits - 5);  // 1024 words = 4 KB: a bin's bitmap, per wave
constexpr int kWordsPerLane = kBinWords / kWave;   // 16
constexpr uint32_t kBinMask = (1u << kBucketBits) - 1u;
constexpr int kDedupWaves = 16;
constexpr int kWindow = 512;                       // pairs a wave stages in LDS at a time (aliases the bitmap)
constexpr uint64_t kNoEntry = ~0ULL;
constexpr int kUnroll = 8;                         // independent loads a lane keeps in flight while streaming
constexpr int kWaveLdsWords = kBinWords + kBinWords / 2; // bitmap (or pair window) + uint16 prefix per word

size_t dedup_lds_bytes(int32_t nbins) { return (size_t)nbins * 8 + (size_t)kDedupWaves * kWaveLdsWords * 4; }

// mb_edgeoff[i] = first entry of minibatch i in the stacked column array
__global__ void mb_edge_offsets_kernel(const int64_t *__restrict__ out_rowptr, const int64_t *__restrict__ mb_rowoff,
                                       int32_t k, int64_t *mb_edgeoff)
{
    for (int32_t i = blockIdx.x * blockDim.x + threadIdx.x; i <= k; i += gridDim.x * blockDim.x)
        mb_edgeoff[i] = out_rowptr[mb_rowoff[i]];
}

void launch_mb_edge_offsets(hipStream_t stream, const int64_t *rowptr, const int64_t *mb_rowoff, int32_t k,
                            int64_t *mb_edgeoff)
{
    hipLaunchKernelGGL(mb_edge_offsets_kernel, dim3((k + 256) / 256), dim3(256), 0, stream, rowptr, mb_rowoff, k,
                       mb_edgeoff);
}

// entry written for every pair / every distinct id: low 32 bits payload, then rank in group, then bin
__device__ inline uint64_t pack_entry(uint32_t payload, uint32_t rank, uint32_t bin)
{
    return (uint64_t)payload | ((uint64_t)rank << 32) | ((uint64_t)bin << 48);
}

// LDS layout of a wave's bitmap.  Lane l owns the 16 logical words [16 l, 16 l + 16) (ascending
// ids), stored as four 16-byte quarters; quarter q4 of lane l sits at uint4 index q4*64 + l, so the
// per-lane 16-byte accesses of a wave hit consecutive addresses (no bank conflicts).
__device__ inline uint32_t bm_word_index(uint32_t W) { return ((((W >> 2) & 3u) << 6) + (W >> 4)) * 4u + (W & 3u); }
// per-word prefix (uint16): word q of lane l at halfword index q*64 + l
__device__ inline uint32_t pre_index(uint32_t W) { return ((W & 15u) << 6) + (W >> 4); }

// 64-lane bitonic sorting network, ascending by lane
__device__ inline uint32_t wave_sort_u32(uint32_t c, int lane)
{
#pragma unroll
    for (int kk = 2; kk <= kWave; kk <<= 1) {
#pragma unroll
        for (int j = kk >> 1; j > 0; j >>= 1) {
            const uint32_t o = __shfl_xor(c, j, kWave);
            const bool keep_min = ((lane & j) == 0) == ((lane & kk) == 0);
            c = keep_min ? min(c, o) : max(c, o);
        }
    }
    return c;
}

// A bin with more than 64 pairs: bitmap over its 2^15 ids in the wave's LDS.
__device__ inline uint32_t rank_big_bin(uint32_t *wbm, uint16_t *wpre, uint64_t *__restrict__ pairs,
                                        uint64_t *__restrict__ utmp, uint32_t bin, uint32_t s, uint32_t e, int lane)
{
    uint4 *bm4 = reinterpret_cast<uint4 *>(wbm) + lane;
#pragma unroll
    for (int q = 0; q < kWordsPerLane / 4; ++q)
        bm4[q * kWave] = make_uint4(0, 0, 0, 0);
    __builtin_amdgcn_wave_barrier();
    for (uint32_t j = s + lane; j < e; j += kWave) {
        const uint32_t l = (uint32_t)(pairs[j] >> 32) & kBinMask;
        atomicOr(&wbm[bm_word_index(l >> 5)], 1u << (l & 31));
    }
    __builtin_amdgcn_wave_barrier();
    uint32_t w[kWordsPerLane];
    uint32_t mine = 0;
#pragma unroll
    for (int q = 0; q < kWordsPerLane / 4; ++q) {
        const uint4 x = bm4[q * kWave];
        w[4 * q] = x.x;
        w[4 * q + 1] = x.y;
        w[4 * q + 2] = x.z;
        w[4 * q + 3] = x.w;
        mine += __popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w);
    }
    const uint32_t inc = wave_inclusive_scan(mine);
    const uint32_t cnt = __shfl(inc, kWave - 1, kWave);
    uint32_t run = inc - mine;
    const uint32_t id0 = (bin << kBucketBits) + (uint32_t)lane * (kWordsPerLane * 32);
#pragma unroll
    for (int q = 0; q < kWordsPerLane; ++q) {
        wpre[q * kWave + lane] = (uint16_t)run;
        uint32_t x = w[q];
        while (x) {
            const int bit = __ffs(x) - 1;
            x &= x - 1;
            utmp[s + run] = pack_entry(id0 + q * 32 + bit, run, bin);
            ++run;
        }
    }
    for (uint32_t j = s + cnt + lane; j < e; j += kWave)
        utmp[j] = kNoEntry;
    __builtin_amdgcn_wave_barrier();
    for (uint32_t j = s + lane; j < e; j += kWave) {
        const uint64_t p = pairs[j];
        const uint32_t l = (uint32_t)(p >> 32) & kBinMask;
        const uint32_t wi = l >> 5;
        const uint32_t r = wpre[pre_index(wi)] + __popc(wbm[bm_word_index(wi)] & ((1u << (l & 31)) - 1u));
        pairs[j] = pack_entry((uint32_t)p, r, bin);
    }
    __builtin_amdgcn_wave_barrier();
    return cnt;
}

__global__ __launch_bounds__(kDedupWaves *kWave) void nw_dedup_bucket_kernel(DedupArgs a)
{
    extern __shared__ uint32_t lds[];
    __shared__ uint32_t smem[kDedupWaves];
    __shared__ uint32_t carry_s;
    constexpr int NT = kDedupWaves * kWave;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int32_t nb = a.nbuckets;
    uint32_t *cur = lds;        // bin counts -> starts -> ends
    uint32_t *ubase = lds + nb; // distinct ids of a group (at its last bin) -> distinct ids before the bin's group
    uint32_t *wbm = lds + 2 * nb + wave * kWaveLdsWords;
    uint16_t *wpre = reinterpret_cast<uint16_t *>(wbm + kBinWords);
    uint64_t *win = reinterpret_cast<uint64_t *>(wbm); // pair window, aliases the bitmap

    for (int32_t i = blockIdx.x; i < a.k; i += gridDim.x) {
        const int64_t e0 = a.mb_edgeoff[i];
        const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
        int32_t *__restrict__ col = a.col + e0; // in: global ids, out: local column indices
        uint64_t *__restrict__ pairs = a.pairs + e0;
        uint64_t *__restrict__ utmp = a.utmp + e0;

        // ---- A: partition by id range ----
        for (int32_t b = tid; b < nb; b += NT) {
            cur[b] = 0;
            ubase[b] = 0;
        }
        if (tid == 0)
            carry_s = 0;
        __syncthreads();
        for (uint32_t j0 = 0; j0 < N; j0 += kUnroll * NT) {
            uint32_t g[kUnroll];
#pragma unroll
            for (int q = 0; q < kUnroll; ++q) {
                const uint32_t j = j0 + q * NT + tid;
                g[q] = j < N ? (uint32_t)col[j] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int q = 0; q < kUnroll; ++q)
                if (g[q] != 0xFFFFFFFFu)
                    atomicAdd(&cur[g[q] >> kBucketBits], 1u);
        }
        __syncthreads();
        for (int32_t base = 0; base < nb; base += NT) {
            const int32_t b = base + tid;
            const uint32_t v = b < nb ? cur[b] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<uint32_t, NT>(v, smem, total);
            const uint32_t carry = carry_s;
            if (b < nb)
                cur[b] = carry + ex;
            __syncthreads();
            if (tid == 0)
                carry_s = carry + total;
            __syncthreads();
        }
        for (uint32_t j0 = 0; j0 < N; j0 += kUnroll * NT) {
            uint32_t g[kUnroll];
#pragma unroll
            for (int q = 0; q < kUnroll; ++q) {
                const uint32_t j = j0 + q * NT + tid;
                g[q] = j < N ? (uint32_t)col[j] : 0xFFFFFFFFu;
            }
#pragma unroll
            for (int q = 0; q < kUnroll; ++q)
                if (g[q] != 0xFFFFFFFFu) {
                    const uint32_t pos = atomicAdd(&cur[g[q] >> kBucketBits], 1u);
                    pairs[pos] = ((uint64_t)g[q] << 32) | (uint64_t)(j0 + q * NT + tid);
                }
        }
        __syncthreads(); // cur[b] is now the end of bin b; its start is cur[b-1]

        // ---- B: ranks inside groups of bins ----
        // wave w owns the bins whose first pair lies in [w*per, (w+1)*per)
        const uint32_t per = (N + kDedupWaves - 1) / kDedupWaves;
        int32_t b_lo, b_hi;
        {
            // smallest bin b with start(b) >= pos, start(b) = b ? cur[b-1] : 0
            auto first_bin_from = [&](uint32_t pos) -> int32_t {
                if (pos == 0)
                    return 0;
                int32_t lo = 0, hi = nb;
                while (lo < hi) {
                    const int32_t mid = (lo + hi) >> 1;
                    if (cur[mid] < pos)
                        lo = mid + 1;
                    else
                        hi = mid;
                }
                return lo + 1 < nb ? lo + 1 : nb;
            };
            b_lo = first_bin_from((uint32_t)wave * per);
            b_hi = first_bin_from((uint32_t)(wave + 1) * per);
        }
        const uint32_t lim = b_hi > 0 ? cur[b_hi - 1] : 0u; // end of this wave's pairs
        uint32_t win_base = 0, win_end = 0;                  // pairs [win_base, win_end) are staged in `win`
        int32_t bin = b_lo;
        while (bin < b_hi) {
            const uint32_t start = bin ? cur[bin - 1] : 0u;
            const int32_t span = (b_hi - bin) < kWave ? (b_hi - bin) : kWave;
            const uint32_t end_l = lane < span ? cur[bin + lane] : 0xFFFFFFFFu; // ends of the next 64 bins
            const unsigned long long fits = __ballot(lane < span && end_l - start <= (uint32_t)kWave);
            const int nbins = fits == ~0ULL ? kWave : __ffsll((unsigned long long)~fits) - 1;
            if (nbins == 0) {
                // more than 64 pairs in this bin alone
                const uint32_t e = __shfl(end_l, 0, kWave);
                const uint32_t cnt = rank_big_bin(wbm, wpre, pairs, utmp, (uint32_t)bin, start, e, lane);
                if (lane == 0)
                    ubase[bin] = cnt;
                win_base = win_end = 0; // the bitmap overwrote the window
                bin += 1;
                continue;
            }
            const uint32_t m = __shfl(end_l, nbins - 1, kWave) - start; // pairs in bins [bin, bin + nbins)
            if (m > 0) {
                if (start + m > win_end || start < win_base) {
                    // stage the next kWindow pairs: 8 independent loads per lane, then LDS
                    uint64_t v[kWindow / kWave];
#pragma unroll
                    for (int u = 0; u < kWindow / kWave; ++u) {
                        const uint32_t j = start + u * kWave + lane;
                        v[u] = j < lim ? pairs[j] : kNoEntry;
                    }
#pragma unroll
                    for (int u = 0; u < kWindow / kWave; ++u)
                        win[u * kWave + lane] = v[u];
                    win_base = start;
                    win_end = (start + kWindow < lim) ? start + kWindow : lim;
                    __builtin_amdgcn_wave_barrier();
                }
                uint64_t p = kNoEntry;
                if ((uint32_t)lane < m)
                    p = win[start - win_base + lane];
                const uint32_t idx = (uint32_t)p;
                const uint32_t id0 = (uint32_t)bin << kBucketBits;
                uint32_t c = 0xFFFFFFFFu;
                if ((uint32_t)lane < m)
                    c = ((((uint32_t)(p >> 32)) - id0) << 6) | (uint32_t)lane; // < 64 bins * 2^15 ids * 64
                c = wave_sort_u32(c, lane);
                const bool valid = (uint32_t)lane < m; // the m real entries sort to the front
                const uint32_t rel = c >> 6;
                const uint32_t prev = __shfl_up(rel, 1, kWave);
                const bool head = valid && (lane == 0 || rel != prev);
                const unsigned long long heads = __ballot(head);
                const uint32_t r = (uint32_t)__popcll(heads & ((2ULL << lane) - 1ULL)) - 1u;
                const uint32_t cnt = (uint32_t)__popcll(heads);
                const uint32_t oidx = __shfl(idx, (int)(c & 63u), kWave);
                if (valid)
                    pairs[start + lane] = pack_entry(oidx, r, (uint32_t)bin);
                if (head)
                    utmp[start + r] = pack_entry(id0 + rel, r, (uint32_t)bin);
                if (valid && (uint32_t)lane >= cnt)
                    utmp[start + lane] = kNoEntry; // slots [cnt, m) of the group hold no distinct id
                if (lane == 0)
                    ubase[bin + nbins - 1] = cnt;
            }
            bin += nbins;
        }
        if (tid == 0)
            carry_s = 0;
        __syncthreads();
        for (int32_t base = 0; base < nb; base += NT) {
            const int32_t b = base + tid;
            const uint32_t v = b < nb ? ubase[b] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<uint32_t, NT>(v, smem, total);
            const uint32_t carry = carry_s;
            if (b < nb)
                ubase[b] = carry + ex;
            __syncthreads();
            if (tid == 0)
                carry_s = carry + total;
            __syncthreads();
        }
        if (tid == 0)
            a.mb_count[i] = carry_s;
        // the bases go to global memory for the fix-up kernel
        for (int32_t b = tid; b < nb; b += NT)
            a.bin_base[(int64_t)i * a.stride + b] = ubase[b];
        __syncthreads(); // the next minibatch reuses cur / ubase
    }
}

// ---------------------------------------------------------------------------------------------
// Fix-up (all compute units).  The entries left by the ranking kernel carry (bin, rank in group,
// position in the minibatch); local column = base[bin] + rank has to land at that position.
// Positions are random, and one scattered 4-byte store per sampled edge is bound by the request
// rate of the memory pipeline, so the values travel in two coalesced steps instead:
//   split  a tile of 2048 entries is counting-sorted in LDS by destination range (8192 positions)
//          and every range's run is appended to that range's slot list with wide stores;
//   place  one workgroup per range reads its slot list, scatters the values inside a 32 KB LDS
//          tile and writes the tile out contiguously.
// Minibatches with more than 256 ranges (2 M sampled edges) store directly.
// ---------------------------------------------------------------------------------------------
constexpr int kPlaceTile = 8192;
constexpr int kPlaceShift = 13;
constexpr int kSplitTile = 2048;
constexpr int kMaxPlaceTiles = 256;
static_assert(kPlaceTile == kDedupPlaceTile && (1 << kPlaceShift) == kPlaceTile && kSplitTile == kDedupSplitTile,
              "tile constants out of step");

__global__ __launch_bounds__(256) void nw_dedup_split_kernel(DedupArgs a)
{
    __shared__ uint64_t stage[kSplitTile];
    __shared__ uint32_t cnt[kMaxPlaceTiles], off[kMaxPlaceTiles], gpos[kMaxPlaceTiles];
    __shared__ uint32_t smem[4];
    const int tid = threadIdx.x;
    const int64_t nunits = a.split_tileoff[a.k];
    for (int64_t unit = blockIdx.x; unit < nunits; unit += gridDim.x) {
        const int i = locate_segment(a.split_tileoff, a.k, unit);
        const int64_t e0 = a.mb_edgeoff[i];
        const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
        const uint32_t Q = (N + kPlaceTile - 1) >> kPlaceShift;
        const uint32_t j0 = (uint32_t)(unit - a.split_tileoff[i]) * kSplitTile;
        const uint32_t jend = (j0 + kSplitTile < N) ? j0 + kSplitTile : N;
        const uint64_t *__restrict__ pairs = a.pairs + e0;
        uint64_t ent[kSplitTile / 256];
#pragma unroll
        for (int q = 0; q < kSplitTile / 256; ++q) {
            const uint32_t j = j0 + q * 256 + tid;
            ent[q] = j < jend ? pairs[j] : kNoEntry; // (bin, rank, position)
        }
        if (Q > kMaxPlaceTiles) { // uniform for the workgroup
            int32_t *__restrict__ col = a.col + e0;
            const uint32_t *__restrict__ base = a.bin_base + (int64_t)i * a.stride;
#pragma unroll
            for (int q = 0; q < kSplitTile / 256; ++q)
                if (ent[q] != kNoEntry)
                    col[(uint32_t)ent[q]] = (int32_t)(base[ent[q] >> 48] + (uint32_t)((ent[q] >> 32) & 0xFFFFu));
            continue;
        }
        cnt[tid] = 0;
        __syncthreads();
        uint32_t lpos[kSplitTile / 256];
#pragma unroll
        for (int q = 0; q < kSplitTile / 256; ++q)
            if (ent[q] != kNoEntry)
                lpos[q] = atomicAdd(&cnt[(uint32_t)ent[q] >> kPlaceShift], 1u);
        __syncthreads();
        const uint32_t mine = cnt[tid];
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<uint32_t, 256>(mine, smem, total);
        off[tid] = ex;
        if (mine)
            gpos[tid] = atomicAdd(&a.place_cursor[a.place_tileoff[i] + tid], mine);
        __syncthreads();
#pragma unroll
        for (int q = 0; q < kSplitTile / 256; ++q)
            if (ent[q] != kNoEntry)
                stage[off[(uint32_t)ent[q] >> kPlaceShift] + lpos[q]] = ent[q];
        __syncthreads();
        uint64_t *__restrict__ back = a.back + e0;
        for (uint32_t sidx = tid; sidx < jend - j0; sidx += 256) {
            const uint64_t e = stage[sidx];
            const uint32_t r = (uint32_t)e >> kPlaceShift;
            back[r * kPlaceTile + gpos[r] + (sidx - off[r])] = e;
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void nw_dedup_place_kernel(DedupArgs a)
{
    __shared__ int32_t tile[kPlaceTile];
    const int tid = threadIdx.x;
    const int64_t ntiles = a.place_tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(a.place_tileoff, a.k, t);
        const int64_t e0 = a.mb_edgeoff[i];
        const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
        if (((N + kPlaceTile - 1) >> kPlaceShift) > (uint32_t)kMaxPlaceTiles)
            continue; // stored directly by the split kernel
        const uint32_t p0 = (uint32_t)(t - a.place_tileoff[i]) * kPlaceTile;
        const uint32_t n = (p0 + kPlaceTile < N) ? kPlaceTile : N - p0;
        const uint32_t *__restrict__ base = a.bin_base + (int64_t)i * a.stride;
        const uint64_t *__restrict__ back = a.back + e0 + p0;
        for (uint32_t s0 = 0; s0 < n; s0 += 8 * 256) {
            uint64_t e[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const uint32_t sidx = s0 + q * 256 + tid;
                e[q] = sidx < n ? back[sidx] : kNoEntry;
            }
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (e[q] != kNoEntry) // local column = distinct ids before the entry's bin or segment + its rank there
                    tile[(uint32_t)e[q] & (kPlaceTile - 1)] =
                        (int32_t)(base[e[q] >> 48] + (uint32_t)((e[q] >> 32) & 0xFFFFu));
        }
        __syncthreads();
        int32_t *__restrict__ col = a.col + e0 + p0;
        for (uint32_t sidx = tid; sidx < n; sidx += 256)
            col[sidx] = tile[sidx];
        __syncthreads();
    }
}

// distinct ids to their final place in the next frontier (blockIdx.y = minibatch)
__global__ __launch_bounds__(256) void nw_dedup_front_kernel(DedupArgs a, const int64_t *__restrict__ mb_coloff,
                                                             int32_t *__restrict__ col_vertex)
{
    const int32_t i = blockIdx.y;
    const int64_t e0 = a.mb_edgeoff[i];
    const uint32_t *__restrict__ base = a.bin_base + (int64_t)i * a.stride;
    int32_t *__restrict__ front = col_vertex + mb_coloff[i];
    if (a.C > 0) {
        if (*a.fallback)
            return; // the hop is repeated with the per-minibatch kernel
        // segment path: segment c left its distinct ids, in rank order, at the head of its slots; the minibatch's
        // columns are those lists one after the other.  Walked by destination, 512 columns per wave and step, so the
        // work is even whatever the segments' lengths: the segment of a column is found in the segments' bases (LDS)
        extern __shared__ uint32_t front_lds[]; // base[C + 1], then the segments' first slots
        uint32_t *base_l = front_lds, *soff_l = front_lds + a.C + 1;
        const uint32_t *__restrict__ uids = a.uids + e0;
        const uint32_t *__restrict__ soff = a.seg_off + (int64_t)i * (a.C + 1);
        const uint32_t U = (uint32_t)a.mb_count[i];
        for (int32_t c = threadIdx.x; c < a.C; c += 256) {
            base_l[c] = base[c];
            soff_l[c] = soff[c];
        }
        if (threadIdx.x == 0)
            base_l[a.C] = U;
        __syncthreads();
        const int lane = threadIdx.x & (kWave - 1);
        const uint32_t wv = blockIdx.x * 4 + threadIdx.x / kWave, nwv = gridDim.x * 4;
        for (uint32_t d0 = wv * (8 * kWave); d0 < U; d0 += nwv * (8 * kWave)) {
            // last segment c with base[c] <= d (segments without distinct ids share their base with the next one)
            uint32_t d = d0 + lane;
            int32_t c = 0;
            if (d < U) {
                int32_t hi = a.C;
                while (hi - c > 1) {
                    const int32_t mid = (c + hi) >> 1;
                    if (base_l[mid] <= d)
                        c = mid;
                    else
                        hi = mid;
                }
            }
            uint32_t v[8]; // 8 independent loads in flight per lane
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                d = d0 + u * kWave + lane;
                v[u] = 0;
                if (d < U) {
                    while (base_l[c + 1] <= d) // the lane's columns ascend: the segment only moves forward
                        ++c;
                    v[u] = uids[soff_l[c] + (d - base_l[c])];
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                d = d0 + u * kWave + lane;
                if (d < U)
                    front[d] = (int32_t)v[u];
            }
        }
        return;
    }
    const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
    const uint64_t *__restrict__ utmp = a.utmp + e0;
    for (uint32_t j0 = blockIdx.x * (8 * 256); j0 < N; j0 += gridDim.x * (8 * 256)) {
        uint64_t u[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t j = j0 + q * 256 + threadIdx.x;
            u[q] = j < N ? utmp[j] : kNoEntry;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (u[q] != kNoEntry)
                front[base[u[q] >> 48] + (uint32_t)((u[q] >> 32) & 0xFFFFu)] = (int32_t)(uint32_t)u[q];
    }
}

// EXTRACT of a hop by the per-minibatch kernel (C == 0)
int launch_nw_dedup_bucket(const Launch &L, const DedupArgs &a, const int64_t *out_rowptr, const int64_t *mb_rowoff,
                           int64_t *mb_coloff, int32_t *col_vertex, int64_t *ncols_out, int64_t nnz, const StageMark &mark)
{
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(nw_dedup_bucket_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 128) != hipSuccess)
            (void)hipGetLastError(); // not required on every runtime; the launch below reports real failures
        attr_set = true;
    }
    mark("dd_bins");
    hipLaunchKernelGGL(mb_edge_offsets_kernel, dim3((a.k + 256) / 256), dim3(256), 0, L.stream, out_rowptr, mb_rowoff,
                       a.k, a.mb_edgeoff);
    hipLaunchKernelGGL(nw_dedup_bucket_kernel, dim3(a.k), dim3(kDedupWaves * kWave), dedup_lds_bytes(a.nbuckets),
                       L.stream, a);
    if (hipGetLastError() != hipSuccess)
        return -1;
    launch_offsets_from_counts(L, a.mb_count, a.k, mb_coloff, ncols_out);
    mark("dd_front");
    launch_nw_dedup_front(L, a, mb_coloff, col_vertex, nnz);
    mark("dd_back_split");
    launch_plan_tiles(L, a.mb_edgeoff, a.k, kSplitTile, a.split_tileoff);
    launch_plan_tiles(L, a.mb_edgeoff, a.k, kPlaceTile, a.place_tileoff);
    (void)hipMemsetAsync(a.place_cursor, 0, (size_t)(nnz / kPlaceTile + a.k + 1) * sizeof(uint32_t), L.stream);
    hipLaunchKernelGGL(nw_dedup_split_kernel, dim3(grid_for(L, nnz / kSplitTile + a.k, 8)), dim3(256), 0, L.stream, a);
    mark("dd_place");
    hipLaunchKernelGGL(nw_dedup_place_kernel, dim3(grid_for(L, nnz / kPlaceTile + a.k, 4)), dim3(256), 0, L.stream, a);
    return 0;
}

void launch_nw_dedup_front(const Launch &L, const DedupArgs &a, const int64_t *mb_coloff, int32_t *col_vertex, int64_t nnz)
{
    int gx = (int)((nnz / a.k + 2047) / 2048) + 1; // about one workgroup per 2048 entries of a minibatch
    if (gx > 64)
        gx = 64;
    hipLaunchKernelGGL(nw_dedup_front_kernel, dim3(gx, a.k), dim3(256), (2 * (size_t)a.C + 1) * sizeof(uint32_t), L.stream, a,
                       mb_coloff, col_vertex);
}

} // namespace bms
