// EXTRACT for the node-wise sampler, fast path (Sec. 4.1.3: "remove empty columns"): every
// minibatch's sampled ids are cut into C id ranges ("segments") small enough to be sorted inside
// LDS, so that all random accesses of the dedup happen in LDS and global memory only sees
// coalesced traffic.  All kernels run on every compute unit, whatever the number of minibatches.
//
//   count  per tile of 16384 sampled ids: LDS histogram over the C segments -> global counts
//   scan   per minibatch: segment offsets; raises the fallback flag when a segment would not
//          fit in LDS (ids crowded into a narrow range) -- then these kernels do nothing and the
//          per-minibatch kernel of kernels_dedup.hip does the hop instead
//   split  per tile: counting sort by segment in LDS, every segment's run appended with wide stores
//   sort   per (minibatch, segment): the pairs are sorted by id -- up to 1024 pairs by one wave in
//          registers (bitonic network; more pairs: ranked by a workgroup through a bitmap in LDS); head flags + scan give
//          the rank among the segment's distinct ids; every pair becomes (segment, rank,
//          position), the distinct ids are written in rank order at the head of the segment's slots
//   base   per minibatch: scan of the segments' distinct counts
// The fix-up kernels of kernels_dedup.hip then add the bases and put everything in place.
#include "bms_device.h"
#include "bms_internal.h"

namespace bms {

constexpr uint64_t kNoEntry = ~0ULL;

__device__ inline uint64_t pack_entry(uint32_t payload, uint32_t rank, uint32_t seg)
{
    return (uint64_t)payload | ((uint64_t)rank << 32) | ((uint64_t)seg << 48);
}

template <int TILE, int NT>
__global__ __launch_bounds__(NT) void dd_count_kernel(DedupArgs a, const int64_t *__restrict__ tileoff)
{
    __shared__ uint32_t hist[kMaxSegments];
    const int tid = threadIdx.x;
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
                atomicAdd(&hist[g[q] >> a.cshift], 1u);
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

// one workgroup per minibatch: seg_off = exclusive scan of the counts (C+1 entries), cursors zeroed
__global__ __launch_bounds__(256) void dd_seg_scan_kernel(DedupArgs a)
{
    __shared__ uint32_t smem[4];
    __shared__ uint32_t carry_s;
    const int i = blockIdx.x, tid = threadIdx.x;
    const uint32_t *__restrict__ cnt = a.seg_cnt + (int64_t)i * a.C;
    uint32_t *__restrict__ off = a.seg_off + (int64_t)i * (a.C + 1);
    if (tid == 0)
        carry_s = 0;
    __syncthreads();
    bool too_big = false;
    for (int base = 0; base < a.C; base += 256) {
        const int c = base + tid;
        const uint32_t v = c < a.C ? cnt[c] : 0u;
        too_big |= v > (uint32_t)kSegCap;
        // too many pairs for one wave: listed for the workgroup sort; 513..1024: listed for the wide wave sort
        wave_append(a.big_list, a.big_count, v > 1024u && v <= (uint32_t)kSegCap, (uint32_t)(i * a.C + c));
        wave_append(a.wide_list, a.wide_count, v > 512u && v <= 1024u, (uint32_t)(i * a.C + c));
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

// TILE sampled ids per workgroup step, NT threads.  The larger the tile, the longer the run every segment gets
// in one step (a step's entries spread over all C segments), i.e. the wider the stores.
template <int TILE, int NT>
__global__ __launch_bounds__(NT) void dd_split_kernel(DedupArgs a, const int64_t *__restrict__ tileoff)
{
    extern __shared__ uint64_t split_lds[]; // stage[TILE]; then 3 C words: per-segment count, start in the tile, start in global
    __shared__ uint32_t smem[NT / kWave];
    __shared__ uint32_t carry_s;
    if (*a.fallback)
        return;
    uint64_t *stage = split_lds;
    uint32_t *cnt = reinterpret_cast<uint32_t *>(split_lds + TILE), *off = cnt + a.C, *gpos = cnt + 2 * a.C;
    const int tid = threadIdx.x;
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
        uint64_t ent[TILE / NT];
        uint32_t lpos[TILE / NT];
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q) {
            const uint32_t j = j0 + q * NT + tid;
            ent[q] = j < jend ? (((uint64_t)(uint32_t)col[j] << 32) | (uint64_t)j) : kNoEntry;
        }
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q)
            if (ent[q] != kNoEntry)
                lpos[q] = atomicAdd(&cnt[(uint32_t)(ent[q] >> 32) >> a.cshift], 1u);
        __syncthreads();
        for (int base = 0; base < a.C; base += NT) {
            const int c = base + tid;
            const uint32_t v = c < a.C ? cnt[c] : 0u;
            uint32_t total;
            const uint32_t ex = block_exclusive_scan<uint32_t, NT>(v, smem, total);
            const uint32_t carry = carry_s;
            if (c < a.C) {
                off[c] = carry + ex;
                if (v)
                    gpos[c] = a.seg_off[(int64_t)i * (a.C + 1) + c] + atomicAdd(&a.seg_cursor[(int64_t)i * a.C + c], v);
            }
            __syncthreads();
            if (tid == 0)
                carry_s = carry + total;
            __syncthreads();
        }
#pragma unroll
        for (int q = 0; q < TILE / NT; ++q)
            if (ent[q] != kNoEntry)
                stage[off[(uint32_t)(ent[q] >> 32) >> a.cshift] + lpos[q]] = ent[q];
        __syncthreads();
        uint64_t *__restrict__ pairs = a.pairs + e0;
        for (uint32_t sidx = tid; sidx < jend - j0; sidx += NT) {
            const uint64_t e = stage[sidx];
            const uint32_t c = (uint32_t)(e >> 32) >> a.cshift;
            pairs[gpos[c] + (sidx - off[c])] = e;
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// One wave per (minibatch, segment) of at most 1024 pairs: the sort runs in registers.
// Sort key = (id - first id of the segment) << 12 | slot, 32 bits (segments span <= 2^20 ids).
// Lane l holds sorted positions [16 l, 16 l + 16): compare-exchanges at distance < 16 stay inside
// a lane, larger distances pair the same register of two lanes (one cross-lane move each).
// ---------------------------------------------------------------------------------------------
constexpr int kWaveSeg = 1024; // pairs per segment handled by one wave
constexpr int kRanges = 256;    // destination ranges per minibatch the fused back-split handles (kMaxPlaceTiles)
constexpr int kRangeShift = 13; // 8192 positions per destination range (kDedupPlaceTile)
constexpr int kRangeSize = 1 << kRangeShift;
static_assert(kRangeSize == kDedupPlaceTile && 3 * kRanges <= kWaveSeg, "range constants out of step");
// LDS staging index: lanes that hold neighbouring runs of slots would all hit the same banks
__device__ inline uint32_t swz(uint32_t x) { return x ^ ((x >> 5) & 31u); }

// Value of lane (l ^ MASK) for a power-of-two MASK.  Partners up to 8 lanes away come through the vector
// unit's lane-permute paths (quad permutes, row shifts and rotates: no LDS traffic); 16 and 32 lanes away through
// the LDS crossbar.
template <int MASK>
__device__ inline uint32_t lane_xor(uint32_t x)
{
    if constexpr (MASK == 1) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
    } else if constexpr (MASK == 2) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, true);
    } else if constexpr (MASK == 4) {
        // lanes 0-3 and 8-11 of every row of 16 take the lane 4 above, the others the lane 4 below
        int o = __builtin_amdgcn_update_dpp((int)x, (int)x, 0x104 /* row_shl:4 */, 0xF, 0x5, false);
        o = __builtin_amdgcn_update_dpp(o, (int)x, 0x114 /* row_shr:4 */, 0xF, 0xA, false);
        return (uint32_t)o;
    } else if constexpr (MASK == 8) {
        return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x128 /* row_ror:8 */, 0xF, 0xF, true);
    } else {
        return (uint32_t)__shfl_xor((int)x, MASK, kWave);
    }
}

// Bitonic network over 64*R values, R per lane; lane l ends up with sorted positions [R l, R l + R).
template <int R>
__device__ inline void wave_sort(uint32_t (&c)[R], int lane)
{
#pragma unroll
    for (int size = 2; size <= kWave * R; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            if (stride >= R) {
                const int lmask = stride / R;
                const bool lower = (lane & lmask) == 0;
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const uint32_t o = lmask == 1 ? lane_xor<1>(c[r]) : lmask == 2 ? lane_xor<2>(c[r])
                                     : lmask == 4 ? lane_xor<4>(c[r]) : lmask == 8 ? lane_xor<8>(c[r])
                                     : lmask == 16 ? lane_xor<16>(c[r]) : lane_xor<32>(c[r]);
                    const bool asc = ((lane * R + r) & size) == 0; // always true in the last merge
                    c[r] = (lower == asc) ? min(c[r], o) : max(c[r], o);
                }
            } else {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if ((r & stride) == 0) {
                        const uint32_t x = c[r], y = c[r | stride];
                        const uint32_t lo = min(x, y), hi = max(x, y);
                        const bool asc = ((lane * R + r) & size) == 0;
                        c[r] = asc ? lo : hi;
                        c[r | stride] = asc ? hi : lo;
                    }
                }
            }
        }
    }
}

// Sorts one segment of m <= 64 R pairs and writes its entries; returns the number of distinct ids.
// When `back` is not null the entries go straight to the slot lists of their destination ranges
// (the wave counting-sorts them by range in LDS and appends every run with wide stores, see the
// fix-up kernels); otherwise they return to `pairs` for the stand-alone split kernel.
template <int R>
__device__ inline uint32_t rank_segment_wave(uint64_t *__restrict__ pairs, uint32_t *__restrict__ uids, uint32_t m,
                                             uint32_t id0, uint32_t cseg, uint32_t *idx_l, uint64_t *out_l, int lane,
                                             uint64_t *__restrict__ back, uint32_t *__restrict__ range_cursor, int nq)
{
    uint32_t c[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t j = r * kWave + lane;
        c[r] = 0xFFFFFFFFu;
        if (j < m) {
            const uint64_t p = pairs[j];
            idx_l[j] = (uint32_t)p;
            c[r] = (((uint32_t)(p >> 32) - id0) << 12) | j;
        }
    }
    wave_sort<R>(c, lane);
    __builtin_amdgcn_wave_barrier();
    // sorted position e = R lane + r; heads = first occurrence of an id
    const uint32_t last_below = __shfl_up(c[R - 1], 1, kWave);
    uint32_t heads = 0;
    bool head[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t prev = r ? c[r - 1] : last_below;
        const bool first = (r == 0 && lane == 0);
        head[r] = c[r] != 0xFFFFFFFFu && (first || (c[r] >> 12) != (prev >> 12));
        heads += head[r] ? 1u : 0u;
    }
    const uint32_t inc = wave_inclusive_scan(heads);
    const uint32_t cnt = __shfl(inc, kWave - 1, kWave);
    uint32_t rank = inc - heads; // heads before this lane
    if (back == nullptr) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            rank += head[r] ? 1u : 0u;
            if (c[r] != 0xFFFFFFFFu) // back to the slot the pair came from: the order of the pairs is free
                out_l[swz(c[r] & 0xFFFu)] = pack_entry(idx_l[c[r] & 0xFFFu], rank - 1u, cseg);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t j = r * kWave + lane;
            if (j < m)
                pairs[j] = out_l[swz(j)];
        }
    } else {
        uint32_t pidx[R]; // position of the pair in its minibatch; its destination range is pidx >> 13
#pragma unroll
        for (int r = 0; r < R; ++r)
            pidx[r] = c[r] != 0xFFFFFFFFu ? idx_l[c[r] & 0xFFFu] : 0xFFFFFFFFu;
        __builtin_amdgcn_wave_barrier();
        // the position table is no longer needed: its LDS now holds, per destination range, the entry
        // count, the start inside this wave's staging and (start in the slot list - start in the staging)
        uint32_t *cntq = idx_l, *offq = idx_l + kRanges, *gdelta = idx_l + 2 * kRanges;
        for (int u = 0; u < nq; ++u)
            cntq[u * kWave + lane] = 0;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r = 0; r < R; ++r) // the slot number in the key's low bits gives way to the place within the range
            if (pidx[r] != 0xFFFFFFFFu)
                c[r] = (c[r] & ~0xFFFu) | atomicAdd(&cntq[pidx[r] >> kRangeShift], 1u);
        __builtin_amdgcn_wave_barrier();
        uint32_t carry = 0;
        for (int u = 0; u < nq; ++u) { // lane owns range 64 u + lane
            const uint32_t q = u * kWave + lane;
            const uint32_t mine = cntq[q];
            const uint32_t inc_q = wave_inclusive_scan(mine);
            const uint32_t start = carry + inc_q - mine;
            offq[q] = start;
            if (mine)
                gdelta[q] = q * kRangeSize + atomicAdd(&range_cursor[q], mine) - start;
            carry += __shfl(inc_q, kWave - 1, kWave);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            rank += head[r] ? 1u : 0u;
            if (pidx[r] != 0xFFFFFFFFu)
                out_l[swz(offq[pidx[r] >> kRangeShift] + (c[r] & 0xFFFu))] = pack_entry(pidx[r], rank - 1u, cseg);
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const uint32_t t = r * kWave + lane;
            if (t < m) {
                const uint64_t e = out_l[swz(t)];
                back[gdelta[(uint32_t)e >> kRangeShift] + t] = e;
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
    rank = inc - heads;
    uint32_t *ids_l = reinterpret_cast<uint32_t *>(out_l); // the distinct ids in rank order, staged for wide stores
#pragma unroll
    for (int r = 0; r < R; ++r) {
        rank += head[r] ? 1u : 0u;
        if (head[r])
            ids_l[swz(rank - 1u)] = id0 + (c[r] >> 12);
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint32_t j = r * kWave + lane;
        if (j < cnt)
            uids[j] = ids_l[swz(j)];
    }
    __builtin_amdgcn_wave_barrier();
    return cnt;
}

// WIDE = false: segments of at most 512 pairs; WIDE = true: those of 513..1024 pairs, whose sorting
// network needs twice the registers (two kernels, so that the common small segments run at the
// higher occupancy)
template <bool WIDE>
__global__ __launch_bounds__(256) void dd_sort_wave_kernel(DedupArgs a)
{
    constexpr int kIdxWords = WIDE ? kWaveSeg : 3 * kRanges; // per wave; also holds the three range tables
    constexpr int kOutSlots = WIDE ? kWaveSeg : kWaveSeg / 2;
    __shared__ uint32_t idx_all[4 * kIdxWords];  // position of every pair of the segment
    __shared__ uint64_t out_all[4 * kOutSlots];  // staging for coalesced stores
    if (*a.fallback)
        return;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    uint32_t *idx_l = idx_all + wave * kIdxWords;
    uint64_t *out_l = out_all + wave * kOutSlots;
    const int64_t nseg = WIDE ? (int64_t)*a.wide_count : (int64_t)a.k * ((a.C + 3) & ~3);
    for (int64_t w = (int64_t)blockIdx.x * 4 + wave; w < nseg; w += (int64_t)gridDim.x * 4) {
        int64_t i, sg;
        uint32_t cseg;
        if (WIDE) {
            sg = a.wide_list[w];
            i = sg / a.C;
            cseg = (uint32_t)(sg % a.C);
        } else {
            // workgroups that run at the same time take segments of different minibatches, so that their
            // appends to the slot lists do not queue up on the cursors of one minibatch; the 4 waves of a
            // workgroup take neighbouring segments of one minibatch
            const int64_t grp = w >> 2;
            i = grp % a.k;
            cseg = (uint32_t)((grp / a.k) * 4 + (w & 3));
            if (cseg >= (uint32_t)a.C)
                continue;
            sg = i * a.C + cseg;
        }
        const uint32_t *__restrict__ soff = a.seg_off + i * (a.C + 1);
        const uint32_t s0 = soff[cseg], m = soff[cseg + 1] - s0;
        if (m > (uint32_t)kWaveSeg)
            continue; // sorted by a whole workgroup in dd_sort_kernel
        if ((m > 512u) != WIDE)
            continue;
        uint32_t cnt = 0;
        if (m > 0) {
            const int64_t e0 = a.mb_edgeoff[i];
            uint64_t *__restrict__ pairs = a.pairs + e0 + s0;
            uint32_t *__restrict__ uids = reinterpret_cast<uint32_t *>(a.utmp) + e0 + s0;
            const uint32_t id0 = cseg << a.cshift;
            // minibatches of at most 256 destination ranges take the fused back-split
            const uint32_t Ni = (uint32_t)(a.mb_edgeoff[i + 1] - e0);
            const uint32_t Q = (Ni + kRangeSize - 1) >> kRangeShift;
            const bool fused = a.fuse_back && Q <= (uint32_t)kRanges;
            const int nq = (int)((Q + kWave - 1) / kWave); // groups of 64 ranges in use
            uint64_t *back = fused ? a.back + e0 : nullptr;
            uint32_t *cursor = a.place_cursor + a.place_tileoff[i];
            if (WIDE)
                cnt = rank_segment_wave<16>(pairs, uids, m, id0, cseg, idx_l, out_l, lane, back, cursor, nq);
            else if (m <= 64)
                cnt = rank_segment_wave<1>(pairs, uids, m, id0, cseg, idx_l, out_l, lane, back, cursor, nq);
            else if (m <= 128)
                cnt = rank_segment_wave<2>(pairs, uids, m, id0, cseg, idx_l, out_l, lane, back, cursor, nq);
            else if (m <= 256)
                cnt = rank_segment_wave<4>(pairs, uids, m, id0, cseg, idx_l, out_l, lane, back, cursor, nq);
            else
                cnt = rank_segment_wave<8>(pairs, uids, m, id0, cseg, idx_l, out_l, lane, back, cursor, nq);
        }
        if (lane == 0)
            a.seg_cnt[sg] = cnt;
    }
}
template __global__ void dd_sort_wave_kernel<false>(DedupArgs);
template __global__ void dd_sort_wave_kernel<true>(DedupArgs);

// One workgroup per (minibatch, segment) of more than 1024 pairs (ids crowded into the segment's range, or one id
// sampled by many rows): no sort.  The segment spans 2^cshift ids, so a bitmap of that many bits in LDS
// (at most 128 KB) takes every pair's id; the rank of an id among the distinct ones is the number of set bits
// below it (a running count per group of 8 words + popcounts inside the group), the distinct ids in rank
// order are the set bits in order.  The pairs are read twice from memory and never held in LDS, so the
// cost grows with the number of pairs only linearly and a segment may hold up to kSegCap of them
// (the rank field of an entry has 16 bits).
constexpr int kBigThreads = 1024;
constexpr int kRankGroup = 8; // bitmap words per running count
size_t dd_rank_lds_bytes(int cshift)
{
    size_t words = ((size_t)1 << cshift) / 32;
    if (words < (size_t)kRankGroup)
        words = kRankGroup;
    return words * sizeof(uint32_t) + (words / kRankGroup) * sizeof(uint32_t);
}

__global__ __launch_bounds__(kBigThreads) void dd_sort_kernel(DedupArgs a)
{
    extern __shared__ uint32_t rank_lds[]; // bitmap words, then one running count per kRankGroup words
    __shared__ uint32_t smem[kBigThreads / kWave];
    if (*a.fallback)
        return;
    const int tid = threadIdx.x;
    uint32_t nw = (1u << a.cshift) / 32u;
    if (nw < (uint32_t)kRankGroup)
        nw = kRankGroup;
    const uint32_t ng = nw / kRankGroup;
    uint32_t *bm = rank_lds, *before = rank_lds + nw;
    const uint32_t nbig = *a.big_count;
    for (uint32_t x = blockIdx.x; x < nbig; x += gridDim.x) {
        const int64_t sg = a.big_list[x];
        const int64_t i = sg / a.C;
        const uint32_t c = (uint32_t)(sg % a.C);
        const uint32_t *__restrict__ soff = a.seg_off + i * (a.C + 1);
        const uint32_t s0 = soff[c], m = soff[c + 1] - s0;
        const int64_t e0 = a.mb_edgeoff[i];
        uint64_t *__restrict__ pairs = a.pairs + e0 + s0;
        uint32_t *__restrict__ uids = reinterpret_cast<uint32_t *>(a.utmp) + e0 + s0;
        const uint32_t id0 = c << a.cshift;
        for (uint32_t q = tid; q < nw; q += kBigThreads)
            bm[q] = 0;
        __syncthreads();
        for (uint32_t j = tid; j < m; j += kBigThreads) {
            const uint32_t b = (uint32_t)(pairs[j] >> 32) - id0;
            atomicOr(&bm[b >> 5], 1u << (b & 31u));
        }
        __syncthreads();
        // set bits before every group of kRankGroup words: groups dealt to the threads in contiguous runs
        const uint32_t per = (ng + kBigThreads - 1) / kBigThreads;
        const uint32_t g_lo = tid * per, g_hi = (g_lo + per < ng) ? g_lo + per : ng;
        uint32_t mine = 0;
        for (uint32_t g = g_lo; g < g_hi; ++g)
#pragma unroll
            for (int q = 0; q < kRankGroup; ++q)
                mine += __popc(bm[g * kRankGroup + q]);
        uint32_t cnt;
        uint32_t run = block_exclusive_scan<uint32_t, kBigThreads>(mine, smem, cnt);
        for (uint32_t g = g_lo; g < g_hi; ++g) {
            before[g] = run;
            // the distinct ids of this group in rank order
            for (int q = 0; q < kRankGroup; ++q) {
                uint32_t wbits = bm[g * kRankGroup + q];
                while (wbits) {
                    const uint32_t bit = (uint32_t)__ffs((int)wbits) - 1u;
                    uids[run++] = id0 + (g * kRankGroup + q) * 32u + bit;
                    wbits &= wbits - 1u;
                }
            }
        }
        __syncthreads();
        for (uint32_t j = tid; j < m; j += kBigThreads) {
            const uint64_t p = pairs[j];
            const uint32_t b = (uint32_t)(p >> 32) - id0;
            const uint32_t w = b >> 5, g = w / kRankGroup;
            uint32_t rank = before[g] + __popc(bm[w] & ((1u << (b & 31u)) - 1u));
            for (uint32_t q = g * kRankGroup; q < w; ++q)
                rank += __popc(bm[q]);
            pairs[j] = pack_entry((uint32_t)p, rank, c);
        }
        if (tid == 0)
            a.seg_cnt[sg] = cnt;
        __syncthreads();
    }
}

// one workgroup per minibatch: distinct ids before each segment; distinct ids of the minibatch
__global__ __launch_bounds__(256) void dd_base_scan_kernel(DedupArgs a)
{
    __shared__ uint32_t smem[4];
    __shared__ uint32_t carry_s;
    if (*a.fallback)
        return;
    const int i = blockIdx.x, tid = threadIdx.x;
    if (tid == 0)
        carry_s = 0;
    __syncthreads();
    for (int base = 0; base < a.C; base += 256) {
        const int c = base + tid;
        const uint32_t v = c < a.C ? a.seg_cnt[(int64_t)i * a.C + c] : 0u;
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
    if (tid == 0)
        a.mb_count[i] = carry_s;
}

void launch_nw_dedup_sorted(const Launch &L, const DedupArgs &a, int64_t nnz, const StageMark &mark)
{
    mark("dd_count");
    // the flag, the two list counters and the segment counters lie next to each other: one clear
    (void)hipMemsetAsync(a.fallback, 0, (size_t)(a.seg_cnt - reinterpret_cast<uint32_t *>(a.fallback)) * sizeof(uint32_t) +
                                            (size_t)a.k * a.C * sizeof(uint32_t), L.stream);
    (void)hipMemsetAsync(a.place_cursor, 0, (size_t)(nnz / kDedupPlaceTile + a.k + 1) * sizeof(uint32_t), L.stream);
    // tiles of the count / split kernels, of the placing kernel and of the stand-alone back-split
    launch_plan_tiles3(L, a.mb_edgeoff, a.k, kSplitTile16, a.big_tileoff, kDedupPlaceTile, a.place_tileoff, kDedupSplitTile,
                       a.split_tileoff);
    const int64_t tiles = nnz / kSplitTile16 + a.k;
    hipLaunchKernelGGL((dd_count_kernel<kSplitTile16, 1024>), dim3(grid_for(L, tiles, 2)), dim3(1024), 0, L.stream, a,
                       a.big_tileoff);
    hipLaunchKernelGGL(dd_seg_scan_kernel, dim3(a.k), dim3(256), 0, L.stream, a);
    mark("dd_split");
    { // 16384 ids per step, one workgroup of 16 waves per compute unit
        static bool attr_set = false;
        const size_t lds = (size_t)kSplitTile16 * sizeof(uint64_t) + 3 * (size_t)a.C * sizeof(uint32_t);
        if (!attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(dd_split_kernel<kSplitTile16, 1024>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(kSplitTile16 * sizeof(uint64_t) + 3 * kMaxSegments * sizeof(uint32_t))) != hipSuccess)
                (void)hipGetLastError(); // not required on every runtime; a refused launch shows in the caller's error check
            attr_set = true;
        }
        hipLaunchKernelGGL((dd_split_kernel<kSplitTile16, 1024>), dim3(grid_for(L, tiles, 1)), dim3(1024), lds,
                           L.stream, a, a.big_tileoff);
    }
    mark("dd_sort");
    hipLaunchKernelGGL(dd_sort_wave_kernel<false>, dim3(grid_for(L, ((int64_t)a.k * a.C + 3) / 4, 4)), dim3(256), 0, L.stream, a);
    hipLaunchKernelGGL(dd_sort_wave_kernel<true>, dim3(grid_for(L, ((int64_t)a.k * a.C + 3) / 4, 2)), dim3(256), 0, L.stream, a);
    { // segments of more than 1024 pairs: ranked through a bitmap of the segment's id range in LDS
        static bool big_attr_set = false;
        if (!big_attr_set) {
            if (hipFuncSetAttribute(reinterpret_cast<const void *>(dd_sort_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)dd_rank_lds_bytes(20)) != hipSuccess)
                (void)hipGetLastError(); // not required on every runtime; a refused launch shows in the caller's error check
            big_attr_set = true;
        }
        hipLaunchKernelGGL(dd_sort_kernel, dim3(grid_for(L, nnz / 1024 + 1, 2)), dim3(kBigThreads),
                           dd_rank_lds_bytes(a.cshift), L.stream, a);
    }
    hipLaunchKernelGGL(dd_base_scan_kernel, dim3(a.k), dim3(256), 0, L.stream, a);
}

} // namespace bms
