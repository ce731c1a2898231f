// EXTRACT for the node-wise sampler, main path (Sec. 4.1.3: "remove empty columns"): every
// minibatch's sampled ids are cut into C id ranges ("segments") small enough to be ranked inside
// LDS, so that all random accesses of the dedup happen in LDS and global memory only sees
// coalesced traffic.  Positions never travel with the ids: the cut remembers, per position, which
// segment its id went to and where inside the run that its tile appended to that segment, so the
// ranks come back along the same runs.  All kernels run on every compute unit, whatever the
// number of minibatches.
//
//   count    per tile of 8192 positions: LDS histogram over the C segments -> global counts
//   scan     per minibatch: segment offsets; segments too long for one workgroup are listed for the
//            bitmap kernel; raises the fallback flag when a segment fits neither (ids crowded into a
//            narrow range) -- then these kernels do nothing and the per-minibatch kernel of
//            kernels_dedup.hip does the hop instead
//   split    per tile: counting sort by segment in LDS, every segment's run of ids appended to the
//            segment with wide stores; per position (segment, place in run); per (tile, segment)
//            where the run went
//   rank     per (minibatch, segment): a workgroup counts the segment's ids into buckets of about
//            one id (LDS), every id compares itself with the few ids of its bucket, head bits and a
//            popcount prefix give every id its rank among the segment's distinct ids; the distinct
//            ids are written in rank order at the head of the segment's slots
//   bitmap   the listed segments: rank = set bits below the id in a bitmap of the segment's id range
//   base     per minibatch: scan of the segments' distinct counts
//   un-split per tile: the runs' ranks read back with wide loads, base of the segment added, scattered
//            to their positions inside LDS, written out as the tile's local column indices
#include "bms_device.h"
#include "bms_internal.h"

#include <algorithm>

namespace bms {

constexpr int kLocShift = 13; // bits of the place inside a run (a tile holds 2^13 positions)
static_assert(kCutTile == (1 << kLocShift) && kMaxSegments <= (1 << (32 - kLocShift)), "loc word out of step");

// The table of segments of unequal width, copied to LDS by the kernels that look ids up (tab_l: kMaxCells + 1 entries).
__device__ inline void load_seg_table(const DedupArgs &a, uint16_t *tab_l, int nthreads)
{
    if (a.tab == nullptr)
        return;
    for (int x = threadIdx.x; x <= kMaxCells; x += nthreads)
        tab_l[x] = a.tab[x];
    __syncthreads();
}
__device__ inline uint32_t seg_of(const DedupArgs &a, const uint16_t *tab_l, uint32_t id)
{
    return a.tab ? (uint32_t)tab_l[id >> a.fshift] : id >> a.cshift;
}
// first id of segment c and log2 (rounded up) of the number of ids it spans
__device__ inline void seg_range(const DedupArgs &a, uint32_t c, uint32_t &id0, int &wbits)
{
    if (a.tab) {
        const uint32_t f0 = a.seg_first[c], width = (a.seg_first[c + 1] - f0) << a.fshift;
        id0 = f0 << a.fshift;
        wbits = width <= 1u ? 0 : 32 - __clz(width - 1u);
    } else {
        id0 = c << a.cshift;
        wbits = a.cshift;
    }
}

template <int TILE, int NT>
__global__ __launch_bounds__(NT) void dd_count_kernel(DedupArgs a, const int64_t *__restrict__ tileoff)
{
    __shared__ uint32_t hist[kMaxSegments];
    __shared__ uint16_t tab_l[kMaxCells + 1];
    const int tid = threadIdx.x;
    load_seg_table(a, tab_l, NT);
    const int64_t ntiles = tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(tileoff, a.k, t);
        const int64_t e0 = a.mb_edgeoff[i];
        const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
        const uint32_t j0 = (uint32_t)(t - tileoff[i]) * TILE;
        const int32_t *__restrict__ col = a.col + e0;
        for (int c = tid; c < a.C; c += NT)
            hist[c] = 0;
        __syncthreads();
        uint32_t g[TILE / NT];
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q) {
            const uint32_t j = j0 + q * NT + tid;
            g[q] = (j < N && j < j0 + TILE) ? (uint32_t)col[j] : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q)
            if (g[q] != 0xFFFFFFFFu)
                atomicAdd(&hist[seg_of(a, tab_l, g[q])], 1u);
        __syncthreads();
        for (int c = tid; c < a.C; c += NT)
            if (hist[c])
                atomicAdd(&a.seg_cnt[(int64_t)i * a.C + c], hist[c]);
        __syncthreads();
    }
}

// appends `value` of every lane with `flag` to a list in global memory: one atomic per wave
__device__ inline void wave_append(uint32_t *__restrict__ list, uint32_t *__restrict__ count, bool flag, uint32_t value)
{
    const unsigned long long mask = __ballot(flag);
    if (mask == 0)
        return;
    const int lane = threadIdx.x & (kWave - 1);
    const int leader = __ffsll((long long)mask) - 1;
    uint32_t base = 0;
    if (lane == leader)
        base = atomicAdd(count, (uint32_t)__popcll(mask));
    base = __shfl(base, leader, kWave);
    if (flag)
        list[base + __popcll(mask & ((1ull << lane) - 1ull))] = value;
}

constexpr int kRankCapFwd = 4096; // = kRankCap (defined with the ranking kernel below)

// one workgroup per minibatch: seg_off = exclusive scan of the counts (C+1 entries), cursors zeroed
__device__ inline void seg_scan_block(const DedupArgs &a, int i, uint32_t *smem, uint32_t &carry_s)
{
    const int tid = threadIdx.x;
    const uint32_t *__restrict__ cnt = a.seg_cnt + (int64_t)i * a.C;
    uint32_t *__restrict__ off = a.seg_off + (int64_t)i * (a.C + 1);
    if (tid == 0)
        carry_s = 0;
    __syncthreads();
    bool too_big = false;
    for (int base = 0; base < a.C; base += 256) {
        const int c = base + tid;
        const uint32_t v = c < a.C ? cnt[c] : 0u;
        // too many entries for one workgroup of the ranking kernel: listed for the bitmap kernel, which holds the
        // segment's id range as bits in LDS; a segment wider or fuller than that kernel takes sends the hop to the
        // per-minibatch kernel
        const bool big = !a.by_bitmap && v > (uint32_t)kRankCapFwd;
        if (big || v > (uint32_t)kSegCap) {
            uint32_t id0;
            int wbits;
            seg_range(a, (uint32_t)c, id0, wbits);
            too_big |= v > (uint32_t)kSegCap || wbits > a.wbits_max;
        }
        wave_append(a.big_list, a.big_count, big && v <= (uint32_t)kSegCap, (uint32_t)(i * a.C + c));
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<uint32_t, 256>(v, smem, total);
        const uint32_t carry = carry_s;
        if (c < a.C) {
            off[c] = carry + ex;
            a.seg_cursor[(int64_t)i * a.C + c] = 0;
        }
        __syncthreads();
        if (tid == 0)
            carry_s = carry + total;
        __syncthreads();
    }
    if (tid == 0)
        off[a.C] = carry_s;
    if (too_big)
        atomicOr(a.fallback, 1);
}

// Planning of a hop's EXTRACT in one launch.  Workgroup k: first entry of every minibatch in the stacked column
// array (mb_edgeoff[i] = rowptr[mb_rowoff[i]]) and the tiles of the cut (tiles never straddle minibatches).
// Workgroups 0..k-1 (only with `scan`, i.e. when the counts per segment are there already): the segment offsets
// of minibatch i.
__global__ __launch_bounds__(256) void dd_plan_kernel(DedupArgs a, const int64_t *__restrict__ out_rowptr,
                                                      const int64_t *__restrict__ mb_rowoff, int scan)
{
    __shared__ uint32_t smem[4];
    __shared__ uint32_t carry_s;
    __shared__ int64_t smem64[4];
    __shared__ int64_t carry64_s;
    if ((int)blockIdx.x < a.k) {
        if (scan)
            seg_scan_block(a, blockIdx.x, smem, carry_s);
        return;
    }
    const int tid = threadIdx.x;
    if (tid == 0)
        carry64_s = 0;
    __syncthreads();
    for (int32_t base = 0; base < a.k; base += 256) {
        const int32_t i = base + tid;
        int64_t cnt = 0;
        if (i < a.k) {
            const int64_t e0 = out_rowptr[mb_rowoff[i]], e1 = out_rowptr[mb_rowoff[i + 1]];
            a.mb_edgeoff[i] = e0;
            if (i == a.k - 1)
                a.mb_edgeoff[a.k] = e1;
            cnt = (e1 - e0 + kCutTile - 1) / kCutTile;
        }
        int64_t total;
        const int64_t ex = block_exclusive_scan<int64_t, 256>(cnt, smem64, total);
        const int64_t carry = carry64_s;
        if (i < a.k)
            a.big_tileoff[i] = carry + ex;
        __syncthreads();
        if (tid == 0)
            carry64_s = carry + total;
        __syncthreads();
    }
    if (tid == 0)
        a.big_tileoff[a.k] = carry64_s;
}

__global__ __launch_bounds__(256) void dd_seg_scan_kernel(DedupArgs a)
{
    __shared__ uint32_t smem[4];
    __shared__ uint32_t carry_s;
    seg_scan_block(a, blockIdx.x, smem, carry_s);
}

// TILE positions per workgroup step, NT threads.  The larger the tile, the longer the run every segment gets
// in one step (a step's ids spread over all C segments), i.e. the wider the stores.
template <int TILE, int NT>
__global__ __launch_bounds__(NT) void dd_split_kernel(DedupArgs a, const int64_t *__restrict__ tileoff)
{
    extern __shared__ uint32_t split_lds[]; // stage[TILE]; then 3 C words: per-segment count, start in the tile, start in global - start in the tile
    __shared__ uint32_t smem[NT / kWave];
    __shared__ uint32_t carry_s;
    __shared__ uint16_t tab_l[kMaxCells + 1];
    if (*a.fallback)
        return;
    uint32_t *stage = split_lds;
    uint32_t *cnt = split_lds + TILE, *off = cnt + a.C, *gpos = cnt + 2 * a.C;
    const int tid = threadIdx.x;
    load_seg_table(a, tab_l, NT);
    const int64_t ntiles = tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(tileoff, a.k, t);
        const int64_t e0 = a.mb_edgeoff[i];
        const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
        const uint32_t j0 = (uint32_t)(t - tileoff[i]) * TILE;
        const uint32_t jend = (j0 + TILE < N) ? j0 + TILE : N;
        const int32_t *__restrict__ col = a.col + e0;
        for (int c = tid; c < a.C; c += NT)
            cnt[c] = 0;
        if (tid == 0)
            carry_s = 0;
        __syncthreads();
        uint32_t id[TILE / NT];
        uint32_t lpos[TILE / NT]; // segment << kLocShift | place in the tile's run for that segment
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q) {
            const uint32_t j = j0 + q * NT + tid;
            id[q] = j < jend ? (uint32_t)col[j] : 0xFFFFFFFFu; // ids are < 2^31
        }
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q)
            if (id[q] != 0xFFFFFFFFu) {
                const uint32_t c = seg_of(a, tab_l, id[q]);
                lpos[q] = (c << kLocShift) | atomicAdd(&cnt[c], 1u);
            }
        uint32_t *__restrict__ loc = a.loc + e0;
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q)
            if (id[q] != 0xFFFFFFFFu)
                loc[j0 + q * NT + tid] = lpos[q];
        __syncthreads();
        uint32_t *__restrict__ run_gpos = a.run_gpos + t * a.C, *__restrict__ run_cnt = a.run_cnt + t * a.C;
        for (int base = 0; base < a.C; base += NT) {
            const int c = base + tid;
            const uint32_t v = c < a.C ? cnt[c] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<uint32_t, NT>(v, smem, total);
            const uint32_t carry = carry_s;
            if (c < a.C) {
                off[c] = carry + ex;
                uint32_t g = 0;
                if (v)
                    g = a.seg_off[(int64_t)i * (a.C + 1) + c] + atomicAdd(&a.seg_cursor[(int64_t)i * a.C + c], v);
                gpos[c] = g - (carry + ex); // start in global - start in the tile
                run_gpos[c] = g;
                run_cnt[c] = v;
            }
            __syncthreads();
            if (tid == 0)
                carry_s = carry + total;
            __syncthreads();
        }
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q)
            if (id[q] != 0xFFFFFFFFu)
                stage[off[lpos[q] >> kLocShift] + (lpos[q] & (TILE - 1))] = id[q];
        __syncthreads();
        uint32_t *__restrict__ ids_seg = a.ids_seg + e0;
        for (uint32_t sidx = tid; sidx < jend - j0; sidx += NT) {
            const uint32_t g = stage[sidx];
            ids_seg[gpos[seg_of(a, tab_l, g)] + sidx] = g;
        }
        __syncthreads();
    }
}

// One workgroup per (minibatch, segment) of at most kRankCap ids: ranks by counting, no sorting network.
// Every thread keeps its ids (slot j = q NT + tid) in registers through all steps.
//   1  the ids are counted into up to 4096 buckets by their leading bits (about one id per bucket)
//   2  exclusive scan of the bucket sizes (every wave a contiguous part, 16 bytes per lane and access);
//      a bucket of more than kRankMaxInBucket ids (one id sampled by many rows, ids crowded into a narrow range)
//      hands the segment to the bitmap kernel, or the hop to the per-minibatch kernel when the segment is too
//      wide for that
//   3  every id goes to its bucket's place in LDS
//   4  every id looks at the few ids of its bucket: `less` of them are smaller, `eqb` are equal and came before
//      it; with eqb = 0 it is the head of its run of equal ids and sets bit (bucket start + less) = the run's
//      place in ascending order
//   5  popcount prefix over the head bits: the rank of an id among the distinct ones = heads before its run
//   6  ranks leave in slot order; the heads leave their ids at their rank, copied out as the distinct ids
constexpr int kRankCap = 4096;    // ids of a segment that one workgroup of the ranking kernel takes
constexpr int kRankThreads = 512;
constexpr int kRankBucketBits = 12; // at most 4096 buckets
constexpr int kRankMaxInBucket = 32;
static_assert(kRankCap == kRankCapFwd, "segment capacity out of step");

__global__ __launch_bounds__(kRankThreads) void dd_rank_kernel(DedupArgs a)
{
    constexpr int NT = kRankThreads, NW = NT / kWave, PER = kRankCap / NT, NB = 1 << kRankBucketBits;
    __shared__ uint4 cnt4[NB / 4 + 1];           // bucket sizes, then bucket starts; start[nb] = m
    __shared__ uint32_t sorted[kRankCap];        // ids by bucket (relative to the segment's first id); then the distinct ones
    __shared__ uint32_t hbits[kRankCap / 32], hpre[kRankCap / 32];
    __shared__ uint32_t wtot[NW];
    uint32_t *cnt = reinterpret_cast<uint32_t *>(cnt4);
    if (*a.fallback)
        return;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    const int64_t nseg = (int64_t)a.k * a.C;
    // The ids of the segment after this one are fetched while this one is ranked (a workgroup's segments follow one
    // another as chains of dependent steps, and only two workgroups fit a compute unit).
    // where segment w lies: first slot, ids, where its minibatch's ids start
    auto where = [&](int64_t w, uint32_t &s0, uint32_t &m, int64_t &e0) {
        s0 = m = 0;
        e0 = 0;
        if (w < nseg) {
            const int64_t i = w % a.k; // workgroups that run at the same time take segments of different minibatches
            const uint32_t cseg = (uint32_t)(w / a.k);
            const uint32_t *__restrict__ soff = a.seg_off + i * (a.C + 1);
            s0 = soff[cseg];
            m = soff[cseg + 1] - s0;
            e0 = a.mb_edgeoff[i];
        }
    };
    // its ids as the kernel keeps them: slot j = q NT + tid, unused slots all ones (no segment, or one that another
    // kernel ranks: nothing is read)
    auto fetch = [&](uint32_t s0, uint32_t m, int64_t e0, uint32_t (&key)[PER]) {
        const uint32_t *__restrict__ ids = a.ids_seg + e0 + s0;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const uint32_t j = q * NT + tid;
            key[q] = (m <= (uint32_t)kRankCap && j < m) ? ids[j] : 0xFFFFFFFFu;
        }
    };
    uint32_t s0, m, s0_next, m_next;
    int64_t e0, e0_next;
    uint32_t key[PER], key_next[PER];
    where(blockIdx.x, s0, m, e0);
    fetch(s0, m, e0, key);
    for (int64_t w = blockIdx.x; w < nseg; w += gridDim.x, s0 = s0_next, m = m_next, e0 = e0_next) {
        where(w + gridDim.x, s0_next, m_next, e0_next);
        const int64_t i = w % a.k;
        const uint32_t cseg = (uint32_t)(w / a.k);
        const int64_t sg = i * a.C + cseg;
        if (m > (uint32_t)kRankCap || m == 0) { // listed for the bitmap kernel by the scan, or empty
            if (m == 0 && tid == 0)
                a.seg_cnt[sg] = 0;
            fetch(s0_next, m_next, e0_next, key);
            continue;
        }
        uint32_t id0;
        int wbits;
        seg_range(a, cseg, id0, wbits);
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (key[q] != 0xFFFFFFFFu)
                key[q] -= id0;
        // buckets: a power of two >= m, 512..4096, no more than the segment has ids
        int nbits = 32 - __clz(m - 1u); // ceil(log2 m); m = 1: __clz(0) = 32
        if (m == 1u || nbits < 9)
            nbits = 9;
        if (nbits > kRankBucketBits)
            nbits = kRankBucketBits;
        if (nbits > wbits)
            nbits = wbits;
        const int bshift = wbits - nbits;
        const int nb = 1 << nbits;
        const int nqd = nb >= 4 ? nb / 4 : 1;                  // 16-byte quads of counters
        const int qw = (nqd + NW - 1) / NW;                    // per wave
        const int its = (qw + kWave - 1) / kWave;              // per lane: 1 or 2
        for (int qd = tid; qd < nqd; qd += NT)
            cnt4[qd] = make_uint4(0, 0, 0, 0);
        for (uint32_t x = tid; x < (m + 31u) / 32u; x += NT)
            hbits[x] = 0;
        __syncthreads();
        fetch(s0_next, m_next, e0_next, key_next);
        uint32_t slot[PER];
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (key[q] != 0xFFFFFFFFu)
                slot[q] = atomicAdd(&cnt[key[q] >> bshift], 1u);
        __syncthreads();
        // exclusive scan of the bucket sizes, in place
        uint4 cv[2];
        uint32_t inc[2], mine[2];
        uint32_t wave_total = 0;
        bool crowded = false;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            cv[it] = make_uint4(0, 0, 0, 0);
            mine[it] = inc[it] = 0;
            if (it < its) {
                const int lq = it * kWave + lane; // quad inside this wave's part
                if (lq < qw && wave * qw + lq < nqd)
                    cv[it] = cnt4[wave * qw + lq];
                crowded |= cv[it].x > (uint32_t)kRankMaxInBucket || cv[it].y > (uint32_t)kRankMaxInBucket ||
                           cv[it].z > (uint32_t)kRankMaxInBucket || cv[it].w > (uint32_t)kRankMaxInBucket;
                mine[it] = cv[it].x + cv[it].y + cv[it].z + cv[it].w;
                inc[it] = wave_inclusive_scan_dpp(mine[it]) + wave_total;
                wave_total = (uint32_t)__builtin_amdgcn_readlane((int)inc[it], kWave - 1);
            }
        }
        if (lane == 0)
            wtot[wave] = wave_total;
        if (__syncthreads_or(crowded)) { // uniform for the workgroup
            if (tid == 0) {
                if (wbits <= a.wbits_max)
                    a.big_list[atomicAdd(a.big_count, 1u)] = (uint32_t)sg;
                else
                    atomicOr(a.fallback, 1);
            }
#pragma unroll
            for (int q = 0; q < PER; ++q)
                key[q] = key_next[q];
            continue;
        }
        uint32_t run = 0;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2)
            run += w2 < wave ? wtot[w2] : 0u;
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            if (it < its) {
                const int lq = it * kWave + lane;
                if (lq < qw && wave * qw + lq < nqd) {
                    const uint32_t s = run + inc[it] - mine[it];
                    cnt4[wave * qw + lq] = make_uint4(s, s + cv[it].x, s + cv[it].x + cv[it].y, s + cv[it].x + cv[it].y + cv[it].z);
                }
            }
        }
        if (tid == 0)
            cnt[nb] = m;
        __syncthreads();
        uint32_t bs[PER]; // start of the id's bucket; from step 4 on: place of its run
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (key[q] != 0xFFFFFFFFu) {
                bs[q] = cnt[key[q] >> bshift];
                sorted[bs[q] + slot[q]] = key[q];
            }
        __syncthreads();
        // place of every id's run of equal ids in ascending order; heads
        if (bshift == 0) { // one id per bucket: the run is the bucket
#pragma unroll
            for (int q = 0; q < PER; ++q)
                if (key[q] != 0xFFFFFFFFu && slot[q] == 0)
                    atomicOr(&hbits[bs[q] >> 5], 1u << (bs[q] & 31u));
        } else {
#pragma unroll
            for (int q = 0; q < PER; ++q)
                if (key[q] != 0xFFFFFFFFu) {
                    const uint32_t be = cnt[(key[q] >> bshift) + 1u], me = bs[q] + slot[q];
                    uint32_t less = 0, eqb = 0;
                    for (uint32_t t = bs[q]; t < be; ++t) {
                        const uint32_t o = sorted[t];
                        less += o < key[q] ? 1u : 0u;
                        eqb += (o == key[q] && t < me) ? 1u : 0u;
                    }
                    bs[q] += less;
                    slot[q] = eqb; // from here on: 0 marks the head of a run
                    if (eqb == 0)
                        atomicOr(&hbits[bs[q] >> 5], 1u << (bs[q] & 31u));
                }
        }
        __syncthreads();
        const uint32_t nwd = (m + 31u) / 32u; // <= 128 words of head bits
        if (wave == 0) {
            uint32_t carry = 0;
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const uint32_t x = it * kWave + lane;
                const uint32_t pcw = x < nwd ? __popc(hbits[x]) : 0u;
                const uint32_t in2 = wave_inclusive_scan_dpp(pcw) + carry;
                if (x < nwd)
                    hpre[x] = in2 - pcw;
                carry = (uint32_t)__builtin_amdgcn_readlane((int)in2, kWave - 1);
            }
            if (lane == 0) {
                wtot[0] = carry;
                a.seg_cnt[sg] = carry;
            }
        }
        __syncthreads();
        const uint32_t cnt_distinct = wtot[0];
        uint16_t *__restrict__ ranks = a.ranks + e0 + s0;
#pragma unroll
        for (int q = 0; q < PER; ++q)
            if (key[q] != 0xFFFFFFFFu) {
                const uint32_t p = bs[q];
                const uint32_t r = hpre[p >> 5] + __popc(hbits[p >> 5] & ((1u << (p & 31u)) - 1u));
                ranks[q * NT + tid] = (uint16_t)r;
                if (slot[q] == 0)
                    sorted[r] = key[q]; // every id has been looked at (step 4): their place now takes the distinct ones
            }
        __syncthreads();
        uint32_t *__restrict__ uids = a.uids + e0 + s0;
        for (uint32_t r = tid; r < cnt_distinct; r += NT)
            uids[r] = id0 + sorted[r];
#pragma unroll
        for (int q = 0; q < PER; ++q)
            key[q] = key_next[q];
        __syncthreads();
    }
}

// Ranking through a bitmap of the segment's id range in LDS (2^cshift bits, at most 128 KB): no sort.  The rank
// of an id among the segment's distinct ids is the number of set bits below it, the distinct ids in rank order are
// the set bits in order.  Work per segment = one pass over the bitmap (16 bytes per lane and access, no bank
// conflicts) + a few operations per id, whatever the ids' multiplicities; a segment may hold up to kSegCap ids (a
// rank has 16 bits).  LISTED = false: every segment of the hop (hops whose ids are dense enough that the pass over
// the bitmap costs less than sorting); LISTED = true: the segments that the sorting kernel handed over.
//   1  the ids' bits are set (LDS atomics); the first kBmKeep ids of every thread stay in registers
//   2  every wave owns a contiguous part of the bitmap, in "quads" of 128 bits, quad it*64 + lane of the part in
//      iteration it: popcounts, wave totals -> set bits before the wave's part; running count before every quad
//      (16 bits, kept in LDS); the set bits of the quads leave as the distinct ids
//   3  rank of an id = count before its quad + set bits below it inside the quad
//   4  the bitmap is cleared again: word by word through the ids when they are few, else as a whole
constexpr int kBmThreads = 1024;
constexpr int kBmWaves = kBmThreads / kWave;
constexpr int kBmKeep = 4;  // ids per thread kept in registers between the passes (segments up to 4096 ids)
constexpr int kBmIts = 8;   // quads per lane: 16 waves x 64 lanes x 8 quads x 128 bits = 2^20 bits
static_assert(kBmWaves * kWave * kBmIts * 128 == (1 << kMaxBitmapShift), "bitmap geometry out of step");
size_t dd_bitmap_lds_bytes(int cshift)
{
    size_t quads = ((size_t)1 << cshift) / 128;
    if (quads < (size_t)kBmWaves * kWave)
        quads = (size_t)kBmWaves * kWave; // every lane owns at least one quad
    return quads * 16 + quads * sizeof(uint16_t);
}

template <bool LISTED>
__global__ __launch_bounds__(kBmThreads) void dd_bitmap_kernel(DedupArgs a)
{
    extern __shared__ uint4 bm_lds[]; // quads, then one 16-bit running count per quad
    __shared__ uint32_t wtot[kBmWaves];
    if (*a.fallback || a.wbits_max > kMaxBitmapShift)
        return;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    uint32_t nq = (1u << a.wbits_max) / 128u;
    if (nq < (uint32_t)(kBmWaves * kWave))
        nq = kBmWaves * kWave;
    const int its = (int)(nq / (kBmWaves * kWave)); // quads per lane: 1, 2, 4 or 8
    uint4 *quads = bm_lds;
    uint32_t *words = reinterpret_cast<uint32_t *>(bm_lds);
    uint16_t *qpre = reinterpret_cast<uint16_t *>(bm_lds + nq);
    const uint32_t q_wave = (uint32_t)wave * (uint32_t)(its * kWave); // first quad of this wave's part
    const int64_t nwork = LISTED ? (int64_t)*a.big_count : (int64_t)a.k * a.C;
    if ((int64_t)blockIdx.x >= nwork)
        return; // usually nothing is listed
    for (int it = 0; it < its; ++it)
        quads[q_wave + it * kWave + lane] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    // a segment's first ids are fetched while the segment before it is worked on
    struct Seg {
        int64_t sg, e0;
        uint32_t s0, m, c, id0;
        uint32_t keep[kBmKeep]; // the first kBmKeep ids of this thread, relative to the segment's first id
    };
    auto fetch = [&](int64_t x, Seg &g) {
        g.m = 0;
        g.sg = -1;
        if (x >= nwork)
            return;
        if (LISTED)
            g.sg = a.big_list[x];
        else // workgroups that run at the same time take segments of different minibatches
            g.sg = (x % a.k) * a.C + x / a.k;
        const int64_t i = g.sg / a.C;
        g.c = (uint32_t)(g.sg % a.C);
        const uint32_t *__restrict__ soff = a.seg_off + i * (a.C + 1);
        g.s0 = soff[g.c];
        g.m = soff[g.c + 1] - g.s0;
        g.e0 = a.mb_edgeoff[i];
        const uint32_t *__restrict__ ids = a.ids_seg + g.e0 + g.s0;
        uint32_t id0;
        int wbits;
        seg_range(a, g.c, id0, wbits);
        g.id0 = id0;
#pragma unroll
        for (int q = 0; q < kBmKeep; ++q) {
            const uint32_t j = q * kBmThreads + tid;
            g.keep[q] = j < g.m ? ids[j] - id0 : 0xFFFFFFFFu;
        }
    };
    Seg nxt;
    fetch(blockIdx.x, nxt);
    for (int64_t x = blockIdx.x; x < nwork; x += gridDim.x) {
        const Seg cur = nxt;
        fetch(x + gridDim.x, nxt);
        const uint32_t m = cur.m;
        if (m == 0) {
            if (tid == 0)
                a.seg_cnt[cur.sg] = 0;
            continue;
        }
        const uint32_t *__restrict__ ids = a.ids_seg + cur.e0 + cur.s0;
        uint16_t *__restrict__ ranks = a.ranks + cur.e0 + cur.s0;
        uint32_t *__restrict__ uids = a.uids + cur.e0 + cur.s0;
        const uint32_t id0 = cur.id0;
        const int64_t sg = cur.sg;
        const uint32_t(&keep)[kBmKeep] = cur.keep;
        // 1: set bits
#pragma unroll
        for (int q = 0; q < kBmKeep; ++q)
            if (keep[q] != 0xFFFFFFFFu)
                atomicOr(&words[keep[q] >> 5], 1u << (keep[q] & 31u));
        for (uint32_t j = kBmKeep * kBmThreads + tid; j < m; j += kBmThreads) {
            const uint32_t b = ids[j] - id0;
            atomicOr(&words[b >> 5], 1u << (b & 31u));
        }
        __syncthreads();
        // 2: counts before every quad, distinct ids
        uint32_t pc[kBmIts], inc[kBmIts];
        uint32_t wave_total = 0;
#pragma unroll
        for (int it = 0; it < kBmIts; ++it) {
            pc[it] = 0;
            inc[it] = 0;
            if (it < its) {
                const uint4 qv = quads[q_wave + it * kWave + lane];
                pc[it] = __popc(qv.x) + __popc(qv.y) + __popc(qv.z) + __popc(qv.w);
                inc[it] = wave_inclusive_scan_dpp(pc[it]) + wave_total; // set bits of this wave's part up to this quad
                wave_total = (uint32_t)__builtin_amdgcn_readlane((int)inc[it], kWave - 1);
            }
        }
        if (lane == 0)
            wtot[wave] = wave_total;
        __syncthreads();
        uint32_t run = 0, cnt = 0; // set bits before this wave's part; in the whole bitmap
#pragma unroll
        for (int w = 0; w < kBmWaves; ++w) {
            const uint32_t t = wtot[w];
            run += w < wave ? t : 0u;
            cnt += t;
        }
#pragma unroll
        for (int it = 0; it < kBmIts; ++it) {
            if (it < its) {
                uint32_t before = run + inc[it] - pc[it];
                qpre[q_wave + it * kWave + lane] = (uint16_t)before;
                if (pc[it]) { // the quad is read again: holding all of them in registers since the first pass costs more
                    const uint32_t first = id0 + (q_wave + it * kWave + lane) * 128u;
                    const uint4 qv = quads[q_wave + it * kWave + lane];
                    const uint32_t xs[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        uint32_t wbits = xs[u];
                        while (wbits) {
                            const uint32_t bit = (uint32_t)__ffs((int)wbits) - 1u;
                            uids[before++] = first + u * 32u + bit;
                            wbits &= wbits - 1u;
                        }
                    }
                }
            }
        }
        if (tid == 0)
            a.seg_cnt[sg] = cnt;
        __syncthreads();
        // 3: ranks
        auto rank_of = [&](uint32_t b) -> uint32_t {
            const uint4 v = quads[b >> 7];
            const uint32_t w = (b >> 5) & 3u, below = (1u << (b & 31u)) - 1u;
            const uint32_t word = w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w;
            return qpre[b >> 7] + (w > 0 ? __popc(v.x) : 0) + (w > 1 ? __popc(v.y) : 0) + (w > 2 ? __popc(v.z) : 0) +
                   __popc(word & below);
        };
#pragma unroll
        for (int q = 0; q < kBmKeep; ++q)
            if (keep[q] != 0xFFFFFFFFu)
                ranks[q * kBmThreads + tid] = (uint16_t)rank_of(keep[q]);
        for (uint32_t j = kBmKeep * kBmThreads + tid; j < m; j += kBmThreads)
            ranks[j] = (uint16_t)rank_of(ids[j] - id0);
        __syncthreads();
        // 4: clear
        if (m * 4u < nq) {
#pragma unroll
            for (int q = 0; q < kBmKeep; ++q)
                if (keep[q] != 0xFFFFFFFFu)
                    words[keep[q] >> 5] = 0u;
            for (uint32_t j = kBmKeep * kBmThreads + tid; j < m; j += kBmThreads)
                words[(ids[j] - id0) >> 5] = 0u;
        } else {
            for (int it = 0; it < its; ++it)
                quads[q_wave + it * kWave + lane] = make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
    }
}

// One workgroup per minibatch: distinct ids before each segment; distinct ids of the minibatch.  The segment
// counters are left all zero for the next hop.  The workgroup that finishes last then turns the minibatches' counts
// into the stacked column offsets (= the next hop's row offsets), the hop's column count, and the next hop's row
// tiles.  When a segment fitted no ranking kernel (flag), the hop's outputs are written as empty: the caller sees the
// flag with the sizes and repeats the call with the per-minibatch kernel on this hop.
__global__ __launch_bounds__(256) void dd_base_scan_kernel(DedupArgs a, int64_t *mb_coloff, int64_t *ncols_out,
                                                           int64_t *next_tileoff /* k + 2 */, uint32_t *done)
{
    __shared__ uint32_t smem[4];
    __shared__ uint32_t carry_s;
    __shared__ int64_t smem64[4];
    __shared__ int64_t carry64_s, carry64b_s;
    __shared__ uint32_t last_s;
    const bool failed = *a.fallback != 0;
    const int i = blockIdx.x, tid = threadIdx.x;
    if (tid == 0)
        carry_s = 0;
    __syncthreads();
    for (int base = 0; base < a.C; base += 256) {
        const int c = base + tid;
        uint32_t v = 0;
        if (c < a.C) {
            v = a.seg_cnt[(int64_t)i * a.C + c];
            a.seg_cnt[(int64_t)i * a.C + c] = 0;
        }
        uint32_t total;
        const uint32_t ex = block_exclusive_scan<uint32_t, 256>(v, smem, total);
        const uint32_t carry = carry_s;
        if (c < a.C)
            a.bin_base[(int64_t)i * a.stride + c] = carry + ex;
        __syncthreads();
        if (tid == 0)
            carry_s = carry + total;
        __syncthreads();
    }
    if (tid == 0) {
        __hip_atomic_store(&a.mb_count[i], failed ? (int64_t)0 : (int64_t)carry_s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        last_s = atomicAdd(done, 1u) == (uint32_t)a.k - 1u ? 1u : 0u;
    }
    __syncthreads();
    if (!last_s)
        return;
    __threadfence();
    if (tid == 0) {
        carry64_s = 0;
        carry64b_s = 0;
        *done = 0; // for the next hop
    }
    __syncthreads();
    int64_t most = 0;
    for (int32_t base = 0; base < a.k; base += 256) {
        const int32_t j = base + tid;
        const int64_t v = j < a.k ? __hip_atomic_load(&a.mb_count[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
        const int64_t tiles = (v + kRowTile - 1) / kRowTile;
        most = tiles > most ? tiles : most;
        int64_t total, total_t;
        const int64_t ex = block_exclusive_scan<int64_t, 256>(v, smem64, total);
        const int64_t ex_t = block_exclusive_scan<int64_t, 256>(tiles, smem64, total_t);
        const int64_t carry = carry64_s, carry_t = carry64b_s;
        if (j < a.k) {
            mb_coloff[j] = carry + ex;
            next_tileoff[j] = carry_t + ex_t;
        }
        __syncthreads();
        if (tid == 0) {
            carry64_s = carry + total;
            carry64b_s = carry_t + total_t;
        }
        __syncthreads();
    }
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) {
        const int64_t o = __shfl_xor(most, d, kWave);
        most = o > most ? o : most;
    }
    if ((tid & (kWave - 1)) == 0)
        smem64[tid / kWave] = most;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            most = smem64[w] > most ? smem64[w] : most;
        mb_coloff[a.k] = carry64_s;
        *ncols_out = carry64_s;
        next_tileoff[a.k] = carry64b_s;
        next_tileoff[a.k + 1] = most;
    }
}

// The cut in reverse: tile t appended, for every segment c, one run of ids to the segment; the ranks of those
// ids lie at the same places.  Per tile: the runs' ranks are read back run by run (wide loads), the distinct
// ids before the segment are added, the value goes to the position that put the id there (scatter inside
// LDS), and the tile's local column indices leave in position order.
template <int TILE, int NT>
__global__ __launch_bounds__(NT) void dd_unsplit_kernel(DedupArgs a, const int64_t *__restrict__ tileoff)
{
    extern __shared__ uint32_t unsplit_lds[]; // stage[TILE], out[TILE]; then 3 C words: start in the tile, start in global - start in the tile, base
    __shared__ uint32_t smem[NT / kWave];
    __shared__ uint32_t carry_s;
    if (*a.fallback)
        return;
    uint32_t *stage = unsplit_lds, *out = unsplit_lds + TILE;
    uint32_t *off = unsplit_lds + 2 * TILE, *delta = off + a.C, *base_l = off + 2 * a.C;
    const int tid = threadIdx.x;
    const int64_t ntiles = tileoff[a.k];
    for (int64_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const int i = locate_segment(tileoff, a.k, t);
        const int64_t e0 = a.mb_edgeoff[i];
        const uint32_t N = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
        const uint32_t j0 = (uint32_t)(t - tileoff[i]) * TILE;
        const uint32_t jend = (j0 + TILE < N) ? j0 + TILE : N;
        const uint32_t *__restrict__ loc = a.loc + e0;
        uint32_t lc[TILE / NT];
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q) {
            const uint32_t j = j0 + q * NT + tid;
            lc[q] = j < jend ? loc[j] : 0xFFFFFFFFu;
        }
        if (tid == 0)
            carry_s = 0;
        __syncthreads();
        const uint32_t *__restrict__ run_gpos = a.run_gpos + t * a.C, *__restrict__ run_cnt = a.run_cnt + t * a.C;
        for (int base = 0; base < a.C; base += NT) {
            const int c = base + tid;
            const uint32_t v = c < a.C ? run_cnt[c] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<uint32_t, NT>(v, smem, total);
            const uint32_t carry = carry_s;
            if (c < a.C) {
                off[c] = carry + ex;
                delta[c] = run_gpos[c] - (carry + ex);
                base_l[c] = a.bin_base[(int64_t)i * a.stride + c];
            }
            __syncthreads();
            if (tid == 0)
                carry_s = carry + total;
            __syncthreads();
        }
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q)
            if (lc[q] != 0xFFFFFFFFu) {
                const uint32_t c = lc[q] >> kLocShift;
                stage[off[c] + (lc[q] & (TILE - 1))] = (c << kLocShift) | (uint32_t)(q * NT + tid);
            }
        __syncthreads();
        const uint16_t *__restrict__ ranks = a.ranks + e0;
        for (uint32_t s0 = 0; s0 < jend - j0; s0 += 4 * NT) { // four independent loads in flight per lane
            uint32_t x[4], r[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t sidx = s0 + u * NT + tid;
                x[u] = sidx < jend - j0 ? stage[sidx] : 0xFFFFFFFFu;
                if (x[u] != 0xFFFFFFFFu) {
                    const uint32_t c = x[u] >> kLocShift;
                    r[u] = base_l[c] + ranks[delta[c] + sidx];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (x[u] != 0xFFFFFFFFu)
                    out[x[u] & (TILE - 1)] = r[u];
        }
        __syncthreads();
        int32_t *__restrict__ col = a.col + e0 + j0;
        for (uint32_t idx = tid; idx < jend - j0; idx += NT)
            col[idx] = (int32_t)out[idx];
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// Segments of unequal width.  Ids that crowd parts of [0, n) (ids sorted by degree put every hub at one end)
// overfill segments of equal width.  The hop's staged ids are sampled (every 8th block of 2048) into a histogram
// over cells of 2^fshift ids; the cells are then dealt to segments in id order so that every segment holds about
// the same share of the sample -- a cell that alone holds more stays a segment of its own, narrow enough for the
// bitmap kernel.  The table is the same for all minibatches of the hop (they sample the same graph), and a
// recycled result keeps it for the next call.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dd_hist_kernel(const int32_t *__restrict__ col, const int64_t *__restrict__ nnz_ptr,
                                                      int32_t fshift, int32_t cells, uint32_t *__restrict__ hist)
{
    __shared__ uint32_t h[kMaxCells + 1];
    const int tid = threadIdx.x;
    for (int x = tid; x <= cells; x += 256)
        h[x] = 0;
    __syncthreads();
    const int64_t nnz = *nnz_ptr;
    for (int64_t b0 = (int64_t)blockIdx.x * 8 * 2048; b0 < nnz; b0 += (int64_t)gridDim.x * 8 * 2048) {
        uint32_t g[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int64_t j = b0 + q * 256 + tid;
            g[q] = j < nnz ? (uint32_t)col[j] : 0xFFFFFFFFu;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (g[q] != 0xFFFFFFFFu)
                atomicAdd(&h[g[q] >> fshift], 1u);
    }
    __syncthreads();
    for (int x = tid; x < cells; x += 256)
        if (h[x])
            atomicAdd(&hist[x], h[x]);
}

// one workgroup: thread t owns cells 4 t .. 4 t + 3
__global__ __launch_bounds__(1024) void dd_table_kernel(const uint32_t *__restrict__ hist, const int64_t *__restrict__ nnz_ptr,
                                                        int32_t k, int32_t cells, int32_t C, int32_t target_per_mb,
                                                        int32_t max_cells, uint16_t *__restrict__ tab,
                                                        uint32_t *__restrict__ seg_first)
{
    __shared__ uint64_t smem[16];
    __shared__ uint32_t smem32[16];
    const int tid = threadIdx.x;
    uint64_t h[4], mine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int cell = 4 * tid + u;
        h[u] = cell < cells ? hist[cell] : 0u;
        mine += h[u];
    }
    uint64_t S;
    uint64_t before = block_exclusive_scan<uint64_t, 1024>(mine, smem, S);
    // ids of the sample per segment: the share target_per_mb has in a minibatch's ids, and never so few that more
    // than C segments come out (breaks forced by the width limit counted in)
    const uint64_t per_mb = (uint64_t)(*nnz_ptr / k) + 1u;
    const int64_t forced = cells / max_cells + 2;
    const uint64_t room = (uint64_t)(C - forced > 1 ? C - forced : 1);
    uint64_t target = S * (uint64_t)target_per_mb / per_mb + 1u;
    if (target < S / room + 1u)
        target = S / room + 1u;
    uint32_t flags = 0, nflag = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int cell = 4 * tid + u;
        if (cell < cells) {
            const uint64_t prev_before = cell ? before - (u ? h[u - 1] : (uint64_t)hist[cell - 1]) : 0u;
            const bool brk = cell == 0 || before / target != prev_before / target || cell / max_cells != (cell - 1) / max_cells;
            flags |= brk ? 1u << u : 0u;
            nflag += brk ? 1u : 0u;
        }
        before += h[u];
    }
    uint32_t nseg;
    uint32_t seg = block_exclusive_scan<uint32_t, 1024>(nflag, smem32, nseg); // segments that start before this thread's cells
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int cell = 4 * tid + u;
        if (cell < cells) {
            if (flags & (1u << u)) {
                seg_first[seg] = (uint32_t)cell;
                ++seg;
            }
            tab[cell] = (uint16_t)(seg - 1u);
        }
    }
    if (tid == 0)
        tab[cells] = (uint16_t)(nseg - 1u); // ids at the very end of the last cell's range never occur; kept in bounds
    for (uint32_t c = nseg + tid; c <= (uint32_t)C; c += 1024)
        seg_first[c] = (uint32_t)cells; // the segments past the last one in use are empty
}

void launch_nw_dedup_table(const Launch &L, const int32_t *col, const int64_t *nnz, int64_t nnz_bound, int64_t n, int32_t k,
                           int32_t fshift, int32_t C, int32_t target_per_mb, int32_t max_wbits, uint32_t *hist,
                           uint16_t *tab, uint32_t *seg_first)
{
    const int32_t cells = (int32_t)(((n > 0 ? n : 1) + (1LL << fshift) - 1) >> fshift); // <= kMaxCells
    int64_t max_cells = max_wbits >= 31 ? (int64_t)cells + 1 : (1LL << (max_wbits > fshift ? max_wbits - fshift : 0));
    if (max_cells > cells)
        max_cells = cells + 1;
    (void)hipMemsetAsync(hist, 0, ((size_t)cells + 1) * sizeof(uint32_t), L.stream);
    hipLaunchKernelGGL(dd_hist_kernel, dim3(grid_for(L, nnz_bound / (8 * 2048) + 1, 2)), dim3(256), 0, L.stream, col, nnz,
                       fshift, cells, hist);
    hipLaunchKernelGGL(dd_table_kernel, dim3(1), dim3(1024), 0, L.stream, hist, nnz, k, cells, C, target_per_mb,
                       (int32_t)max_cells, tab, seg_first);
}

void launch_nw_extract_segments(const Launch &L, const DedupArgs &a, const int64_t *out_rowptr, const int64_t *mb_rowoff,
                                int64_t *mb_coloff, int32_t *col_vertex, int64_t *ncols_out, int64_t *next_tileoff,
                                uint32_t *done, int64_t nnz, bool counted, const StageMark &mark)
{
    mark("dd_plan");
    const int64_t tiles = nnz / kCutTile + a.k;
    hipLaunchKernelGGL(dd_plan_kernel, dim3(a.k + 1), dim3(256), 0, L.stream, a, out_rowptr, mb_rowoff, counted ? 1 : 0);
    if (!counted) {
        hipLaunchKernelGGL((dd_count_kernel<kCutTile, 512>), dim3(grid_for(L, tiles, 4)), dim3(512), 0, L.stream, a,
                           a.big_tileoff);
        hipLaunchKernelGGL(dd_seg_scan_kernel, dim3(a.k), dim3(256), 0, L.stream, a);
    }
    mark("dd_split");
    { // 8192 ids per step, workgroups of 8 waves, several per compute unit
        static bool attr_set = false;
        const size_t lds = (size_t)kCutTile * sizeof(uint32_t) + 3 * (size_t)a.C * sizeof(uint32_t);
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(dd_split_kernel<kCutTile, 512>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(kCutTile * sizeof(uint32_t) + 3 * kMaxSegments * sizeof(uint32_t))) != hipSuccess)
                (void)hipGetLastError(); // not required on every runtime; a refused launch shows in the caller's error check
            attr_set = true;
        }
        hipLaunchKernelGGL((dd_split_kernel<kCutTile, 512>), dim3(grid_for(L, tiles, 4)), dim3(512), lds,
                           L.stream, a, a.big_tileoff);
    }
    mark("dd_rank");
    static bool big_attr_set = false;
    if (!big_attr_set) {
        const int most = (int)dd_bitmap_lds_bytes(kMaxBitmapShift);
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(dd_bitmap_kernel<false>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, most) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(dd_bitmap_kernel<true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, most) != hipSuccess)
            (void)hipGetLastError(); // not required on every runtime; a refused launch shows in the caller's error check
        big_attr_set = true;
    }
    const size_t bm_lds = dd_bitmap_lds_bytes(a.wbits_max <= kMaxBitmapShift ? a.wbits_max : kMaxBitmapShift);
    const int bm_per_cu = (int)std::max<size_t>(1, std::min<size_t>(2, (size_t)(156 * 1024) / bm_lds));
    if (a.by_bitmap) {
        hipLaunchKernelGGL(dd_bitmap_kernel<false>, dim3(grid_for(L, (int64_t)a.k * a.C, bm_per_cu)), dim3(kBmThreads),
                           bm_lds, L.stream, a);
    } else {
        hipLaunchKernelGGL(dd_rank_kernel, dim3(grid_for(L, (int64_t)a.k * a.C, 4)), dim3(kRankThreads), 0, L.stream, a);
        if (a.tab || a.cshift <= kMaxBitmapShift) // segments the counting kernel did not take (none can be listed otherwise)
            hipLaunchKernelGGL(dd_bitmap_kernel<true>, dim3(grid_for(L, nnz / 1024 + 1, bm_per_cu)), dim3(kBmThreads),
                               bm_lds, L.stream, a);
    }
    hipLaunchKernelGGL(dd_base_scan_kernel, dim3(a.k), dim3(256), 0, L.stream, a, mb_coloff, ncols_out, next_tileoff, done);
    mark("dd_front");
    launch_nw_dedup_front(L, a, mb_coloff, col_vertex, nnz);
    mark("dd_unsplit");
    launch_nw_dedup_unsplit(L, a, nnz);
}

void launch_nw_dedup_unsplit(const Launch &L, const DedupArgs &a, int64_t nnz)
{
    static bool attr_set = false;
    const size_t lds = 2 * (size_t)kCutTile * sizeof(uint32_t) + (3 * (size_t)a.C + 1) * sizeof(uint32_t);
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(dd_unsplit_kernel<kCutTile, 512>),
                                hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)(2 * kCutTile * sizeof(uint32_t) + (3 * kMaxSegments + 1) * sizeof(uint32_t))) != hipSuccess)
            (void)hipGetLastError(); // not required on every runtime; a refused launch shows in the caller's error check
        attr_set = true;
    }
    const int64_t tiles = nnz / kCutTile + a.k;
    hipLaunchKernelGGL((dd_unsplit_kernel<kCutTile, 512>), dim3(grid_for(L, tiles, 2)), dim3(512), lds, L.stream, a,
                       a.big_tileoff);
}

} // namespace bms
