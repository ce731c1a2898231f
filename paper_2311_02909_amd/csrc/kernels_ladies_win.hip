// Layer-wise (LADIES) bulk sampling, Sec. 4.2 of arxiv 2311.02909: the path that accumulates the
// column counts of P = Q A in LDS.
//
// The rows of A are sorted by column, so the neighbours of a frontier row that fall into a window
// of 2^16 vertex ids form one contiguous piece of its adjacency list.  One hop, all k minibatches:
//   ldw_plan, ldw_tile_rows
//                   the gathered order (the neighbour lists of the stacked frontier laid end to end) cut into
//                   tiles of 1024..4096 positions (few gathered neighbours: small tiles, so that every wave still
//                   gets some) that never straddle minibatches; the row each tile starts in
//   ldw_bounds      where every row crosses every window boundary (lower bounds, one list per row).  A row's list
//                   depends on its vertex alone: when the lists of all n vertices fit in memory they are computed
//                   once per graph (one wave per tile streams its pieces of rows, the "hop" being the whole
//                   graph) and a hop only copies the lists of its rows; else the hop streams its rows for them.
//                   Either way the lists are turned window-major for the next kernel
//   ldw_win_added   neighbours of every (minibatch, window): the lengths of its pieces added up
//   ldw_accumulate  one workgroup per (minibatch, window): 2^16 packed 16-bit counters in LDS (128 KB); every
//                   row's piece of the window adds 1 per neighbour (e_v cannot exceed the number of frontier
//                   rows, which this path keeps below 2^16); each wave then compacts its sixteenth of the window
//                   (a part): the nonzero counters leave in ascending column order as 4-byte entries
//                   (column - window start, e_v) into room claimed from a device-wide cursor
//   ldw_win_scan    per minibatch: columns and weight of every window, before each of its parts, before the window
//   ldw_p_copy      parts copied to their place in P, one wave per part; inclusive prefix sums of the integer
//                   weights (e_v or e_v^2) on the way, one kept per 16 entries (NORM stays implicit: draws are
//                   integers below the row sum)
//   ldw_draw        SAMPLE (Sec. 4.2.2): one workgroup per minibatch: s draws, each the smallest t
//                   with prefix[t] > r, sorted in LDS, duplicates dropped -> sampled columns
//   ldw_extract     EXTRACT (Sec. 4.2.3): the sampled columns of the minibatch sit in an LDS hash
//                   table (column -> local index); one wave per tile streams the gathered order a
//                   second time and keeps the neighbours found in the table ((Q_R A) Q_C), in
//                   row order, piece by piece; rows are then sized by a scan and their pieces
//                   copied to their place
// A call that sizes its buffers from an earlier call of the same shape runs all of these behind LwHop::giveup.
#include "bms_device.h"
#include "bms_internal.h"
#include <algorithm>

namespace bms {

constexpr int kWinIds = 1 << kWinShift;
constexpr int kWinWords = kWinIds / 2; // two 16-bit counters per LDS word
constexpr int kAccThreads = 1024;
constexpr int kAccWaves = kAccThreads / kWave;
static_assert(kAccWaves == kWinParts, "one part of a window per wave of the accumulation");
constexpr int kWaveWords = kWinWords / kAccWaves; // counter words compacted by one wave
constexpr uint32_t kEmptySlot = 0xFFFFFFFFu;
constexpr int kExtThreads = 1024; // the waves of a workgroup share one hash table
constexpr int kExtWaves = kExtThreads / kWave;
constexpr int kAccUnroll = 8;              // 16-byte loads per lane in flight while a wave gathers
constexpr int kAccChunks = kWave * kAccUnroll; // aligned 16-byte chunks per span: one per lane and load
struct AccPiece {                          // one nonempty piece of a wave's 64 rows
    int64_t origin;                        // byte address of its first line - 128 * lines of the wave before it
    uint32_t lo_rel, hi_rel;               // its bytes, relative to origin
};
constexpr int kStreamUnroll = 8; // neighbours per lane in flight in the two streaming passes
constexpr int kHashSlots = 2 * kMaxWinSampled;    // load factor <= 1/2
constexpr int kDrawTop = 2048;                    // recorded weight sums of P that a drawing workgroup keeps in LDS

__device__ inline uint64_t ldw_weight(uint32_t cnt, int squared)
{
    return squared ? (uint64_t)cnt * (uint64_t)cnt : (uint64_t)cnt;
}

// ---------------------------------------------------------------------------------------------
// Tiles of the gathered order
// ---------------------------------------------------------------------------------------------
// One workgroup: where each minibatch starts in the gathered order (mb_goff), the tiles before each minibatch
// (mb_gtileoff); the tile counters of the extraction and the staging cursor of the accumulation start at zero.
__global__ __launch_bounds__(1024) void ldw_plan_kernel(LwHop a)
{
    __shared__ int64_t smem[16];
    __shared__ int64_t carry_s;
    if (threadIdx.x == 0) {
        carry_s = 0;
        if (a.cursor)
            *a.cursor = 0;
        if (a.giveup && a.gather_off[a.mb_rowoff[a.k]] > a.gathered_cap)
            *a.giveup = 1; // the kernels after this one see it: they are launched after this one ends
    }
    __syncthreads();
    for (int32_t base = 0; base <= a.k; base += 1024) {
        const int32_t i = base + threadIdx.x;
        int64_t cnt = 0;
        if (i <= a.k) {
            const int64_t g0 = a.gather_off[a.mb_rowoff[i]];
            a.mb_goff[i] = g0;
            if (a.tile_queue)
                a.tile_queue[i] = 0;
            if (i < a.k)
                cnt = (a.gather_off[a.mb_rowoff[i + 1]] - g0 + a.tile - 1) / a.tile;
        }
        int64_t total;
        const int64_t ex = block_exclusive_scan<int64_t, 1024>(cnt, smem, total);
        const int64_t carry = carry_s;
        if (i <= a.k)
            a.mb_gtileoff[i] = carry + ex; // entry k: all tiles
        __syncthreads();
        if (threadIdx.x == 0)
            carry_s = carry + total;
        __syncthreads();
    }
}

// tile_row[x] = the row that holds the first position of tile x (the last row starting at or before it)
__global__ __launch_bounds__(256) void ldw_tile_rows_kernel(LwHop a)
{
    if (a.giveup && *a.giveup)
        return;
    const int64_t ntiles = a.mb_gtileoff[a.k];
    for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < ntiles; x += (int64_t)gridDim.x * 256) {
        const int i = locate_segment(a.mb_gtileoff, a.k, x);
        const int64_t g0 = a.mb_goff[i] + (x - a.mb_gtileoff[i]) * a.tile;
        int64_t lo = a.mb_rowoff[i], hi = a.mb_rowoff[i + 1];
        while (hi - lo > 1) {
            const int64_t mid = (lo + hi) >> 1;
            if (a.gather_off[mid] <= g0)
                lo = mid;
            else
                hi = mid;
        }
        a.tile_row[x] = lo;
    }
}

// Walks the pieces of rows inside tile [g0, g1) of the gathered order, starting in row r0 (the row that holds
// g0), and calls body(r, rs, re, shift, g, pe) for each: row r spans gathered positions [rs, re), the piece is
// [g, pe), and A_col[shift + p] is the neighbour at position p.  The extent of the following row is fetched
// while a piece is being worked on, so a new piece does not start with a chain of dependent loads.
template <class Body>
__device__ inline void ldw_walk_tile(const LwHop &a, int64_t g0, int64_t g1, int64_t r0, int64_t nrows, Body body)
{
    int64_t g = g0, r = r0;
    int64_t rs = a.gather_off[r], re = a.gather_off[r + 1], beg = a.row_beg[r];
    while (g < g1) {
        const int64_t rn = r + 1 < nrows ? r + 1 : r;
        const int64_t next_re = a.gather_off[rn + 1], next_beg = a.row_beg[rn];
        const int64_t pe = min(re, g1);
        body(r, rs, re, beg - rs, g, pe);
        g = pe;
        if (pe == re) {
            ++r;
            rs = re;
            re = next_re;
            beg = next_beg;
            while (re <= g && g < g1) { // rows without neighbours
                ++r;
                rs = re;
                re = a.gather_off[r + 1];
                beg = a.row_beg[r];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// bounds[r * (nwin + 1) + w] = number of neighbours of row r with id < w * 2^16, w = 0..nwin (row-major:
// the wave that streams a row writes its boundaries next to each other)
// (rows without neighbours are skipped: their entries are never read)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void ldw_bounds_kernel(LwHop a)
{
    if (a.giveup && *a.giveup)
        return;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t ntiles = a.mb_gtileoff[a.k];
    const int64_t nrows = a.mb_rowoff[a.k];
    for (int64_t x = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave; x < ntiles; x += (int64_t)gridDim.x * 4) {
        const int i = locate_segment(a.mb_gtileoff, a.k, x);
        const int64_t g0 = a.mb_goff[i] + (x - a.mb_gtileoff[i]) * a.tile;
        const int64_t g1 = min(g0 + a.tile, a.mb_goff[i + 1]);
        ldw_walk_tile(a, g0, g1, a.tile_row[x], nrows,
                      [&](int64_t r, int64_t rs, int64_t re, int64_t shift, int64_t g, int64_t pe) {
            uint32_t *__restrict__ out = a.bounds + r * (a.nwin + 1);
            // when the row ends inside the tile, position `re` acts as one more entry that lies in
            // window nwin: it closes every window left
            const int64_t last = pe == re ? pe : pe - 1;
            int32_t carry = g == rs ? -1 : (a.A_col[shift + g - 1] >> kWinShift); // window of the entry before
            for (int64_t p0 = g; p0 <= last; p0 += kStreamUnroll * kWave) {
                // 32-bit slot numbers from here on: slot x of the step is gathered position p0 + x
                const int32_t *__restrict__ from = a.A_col + (shift + p0);
                const int32_t nreal = (int32_t)min<int64_t>(re - p0, kStreamUnroll * kWave); // slots that hold a neighbour
                const int32_t xlast = (int32_t)min<int64_t>(last - p0, kStreamUnroll * kWave - 1);
                const uint32_t pos0 = (uint32_t)(p0 - rs);
                int32_t wv[kStreamUnroll];
#pragma unroll
                for (int u = 0; u < kStreamUnroll; ++u) {
                    const int32_t x = u * kWave + lane;
                    wv[u] = x < nreal && x <= xlast ? (from[x] >> kWinShift) : a.nwin;
                }
#pragma unroll
                for (int u = 0; u < kStreamUnroll; ++u) {
                    const int32_t x = u * kWave + lane;
                    // window of the entry one lane below (lane 0: of the entry before the step): a lane shift in
                    // the vector unit, not a trip through LDS
                    const int32_t pw = __builtin_amdgcn_update_dpp(carry, wv[u], 0x138 /* wave_shr:1 */, 0xF, 0xF, false);
                    if (x <= xlast) // this entry is the first at or past the boundaries pw+1 .. wv
                        for (int32_t w = pw + 1; w <= wv[u]; ++w)
                            out[w] = pos0 + (uint32_t)x;
                    carry = __builtin_amdgcn_readlane(wv[u], kWave - 1);
                }
            }
        });
    }
}

// The boundary lists turned window-major (bounds_t[w * rows_bound + r]): the accumulation reads one window of
// all rows at a time.  64 x 64 tiles through LDS, both sides coalesced.  The list of row r comes from this
// hop's boundary pass, or, when the graph carries an index of every vertex's list, from the index entry of
// the row's vertex.
__global__ __launch_bounds__(256) void ldw_bounds_transpose_kernel(LwHop a)
{
    __shared__ uint32_t tile[64][65];
    if (a.giveup && *a.giveup)
        return;
    const int64_t ncols = a.nwin + 1;
    const int64_t nrows = a.index ? a.mb_rowoff[a.k] : a.rows_bound;
    const int64_t tiles_c = (ncols + 63) / 64, tiles_r = (nrows + 63) / 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int64_t t = blockIdx.x; t < tiles_c * tiles_r; t += gridDim.x) {
        const int64_t r0 = (t / tiles_c) * 64, c0 = (t % tiles_c) * 64;
        if (a.index) { // the rows' vertices first, then all of a thread's 16 reads of the index in flight together
            int64_t v[16];
#pragma unroll
            for (int q = 0; q < 16; ++q)
                v[q] = r0 + ty + 4 * q < nrows ? (int64_t)a.row_vertex[r0 + ty + 4 * q] : -1;
            uint32_t x[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) // a seed outside [0, n) is an error reported elsewhere; its row has no neighbours
                x[q] = (v[q] >= 0 && v[q] < a.n && c0 + tx < ncols) ? a.index[v[q] * ncols + c0 + tx] : 0u;
#pragma unroll
            for (int q = 0; q < 16; ++q)
                tile[ty + 4 * q][tx] = x[q];
        } else {
            for (int y = ty; y < 64; y += 4)
                if (r0 + y < nrows && c0 + tx < ncols)
                    tile[y][tx] = a.bounds[(r0 + y) * ncols + c0 + tx];
        }
        __syncthreads();
        for (int y = ty; y < 64; y += 4)
            if (c0 + y < ncols && r0 + tx < nrows)
                a.bounds_t[(c0 + y) * a.rows_bound + r0 + tx] = tile[tx][y];
        __syncthreads();
    }
}

// win_added[i * nwin + w] = neighbours of minibatch i's rows inside window w (the lengths of their pieces)
__global__ __launch_bounds__(256) void ldw_win_added_kernel(LwHop a)
{
    __shared__ uint32_t wsum[4];
    if (a.giveup && *a.giveup)
        return;
    const int tid = threadIdx.x;
    const int64_t nblk = (int64_t)a.k * a.nwin;
    for (int64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const int i = (int)(blk / a.nwin), w = (int)(blk % a.nwin);
        const uint32_t *__restrict__ lo_b = a.bounds_t + (int64_t)w * a.rows_bound;
        uint32_t sum = 0; // < 2^32: at most 65535 rows with at most 2^16 neighbours in a window each
        for (int64_t r = a.mb_rowoff[i] + tid; r < a.mb_rowoff[i + 1]; r += 256)
            if (a.gather_off[r + 1] != a.gather_off[r]) // rows without neighbours have no boundaries on record
                sum += lo_b[a.rows_bound + r] - lo_b[r];
        sum = wave_sum(sum);
        __syncthreads();
        if ((tid & (kWave - 1)) == 0)
            wsum[tid / kWave] = sum;
        __syncthreads();
        if (tid == 0)
            a.win_added[blk] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
}

// ---------------------------------------------------------------------------------------------
// P = Q A for one (minibatch, window) per workgroup
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kAccThreads) void ldw_accumulate_kernel(LwHop a)
{
    extern __shared__ uint32_t lds[];
    if (a.giveup && *a.giveup)
        return;
    uint32_t *cnt = lds;                   // kWinWords packed counters
    unsigned long long *claim_s = reinterpret_cast<unsigned long long *>(lds + kWinWords); // [2], in turn: where the
                                           // entries of the current (minibatch, window) start in the staging array
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
    // per wave: one record per nonempty piece (by rank) and the start bits of one span of chunks
    AccPiece *piece_rec = reinterpret_cast<AccPiece *>(lds + kWinWords + 3 * kAccWaves + 4) + wave * (kWave + kAccUnroll / 2);
    uint32_t *starts = reinterpret_cast<uint32_t *>(piece_rec + kWave); // kAccChunks bits
    const uint64_t below = (1ull << lane) - 1ull, below_incl = below | (1ull << lane);
    const int64_t A0 = (int64_t)reinterpret_cast<uintptr_t>(a.A_col);
    const int64_t nblk = (int64_t)a.k * a.nwin;
    // the counters start at zero and every (minibatch, window) leaves them at zero: the pass that emits the
    // nonzero ones clears them
    for (int x = tid; x < kWinWords; x += kAccThreads)
        cnt[x] = 0;
    __syncthreads();
    int turn = 0;
    // Workgroups are handed to the chip's 8 dies in turn, and each die has its own last-level cache.  Within a
    // round of gridDim.x (minibatch, window) pairs, die x takes a run of consecutive windows, so the memory
    // lines that hold the end of one window's piece and the start of the next one's are fetched once.
    const int64_t G = gridDim.x;
    const bool by_die = (G % 8) == 0;
    auto block_of = [&](int64_t slot) {
        int64_t blk = slot;
        if (by_die) {
            const int64_t p = slot % G;
            blk = slot - p + (p % 8) * (G / 8) + p / 8;
        }
        return blk;
    };
    // the piece of window w in row r, r < r1: (length, address of its first neighbour); rows without
    // neighbours have no boundaries on record: whatever is read there is dropped
    auto piece_at = [&](int w, int64_t r, int64_t r1, uint32_t &len, int64_t &addr) {
        len = 0;
        addr = 0;
        if (r < r1) {
            const uint32_t *__restrict__ lo_b = a.bounds_t + (int64_t)w * a.rows_bound; // boundary w of every row
            const uint32_t b0 = lo_b[r];
            const uint32_t b1 = lo_b[a.rows_bound + r];
            const bool empty = a.gather_off[r + 1] == a.gather_off[r];
            len = empty ? 0u : b1 - b0;
            addr = a.row_beg[r] + b0;
        }
    };
    // the first pieces of a (minibatch, window) pair are fetched while the pair before it is compacted
    auto first_pieces = [&](int64_t slot, uint32_t &len, int64_t &addr) {
        const int64_t blk = block_of(slot);
        len = 0;
        addr = 0;
        if (blk < nblk) {
            const int i = (int)(blk / a.nwin);
            piece_at((int)(blk % a.nwin), a.mb_rowoff[i] + (int64_t)wave * kWave + lane, a.mb_rowoff[i + 1], len, addr);
        }
    };
    uint32_t len, next_len;
    int64_t addr, next_addr;
    first_pieces(blockIdx.x, len, addr);
    for (int64_t slot = blockIdx.x; slot < (nblk + G - 1) / G * G; slot += G) {
        const int64_t blk = block_of(slot);
        if (blk >= nblk) { // no later slot of this workgroup holds a pair either
            first_pieces(slot + G, len, addr);
            continue;
        }
        const int i = (int)(blk / a.nwin), w = (int)(blk % a.nwin);
        const int64_t r0 = a.mb_rowoff[i], r1 = a.mb_rowoff[i + 1];
        const int32_t id0 = w << kWinShift;
        auto piece_of = [&](int64_t r, uint32_t &l, int64_t &ad) { piece_at(w, r, r1, l, ad); };
        // A part of the window (one wave's kWaveWords words) cannot hold more columns than it has counters, nor
        // than the window gets neighbours: room for that many entries per part is claimed from the device-wide
        // cursor now, and the answer is back long before the counters are compacted
        const uint32_t added_blk = a.win_added[blk];
        const uint32_t room = min(added_blk, (uint32_t)(2 * kWaveWords));
        if (tid == 0)
            claim_s[turn] = room ? atomicAdd(a.cursor, (unsigned long long)room * kWinParts) : 0ull;
        for (int64_t base = r0 + (int64_t)wave * kWave; base < r1; base += (int64_t)kAccWaves * kWave) {
            // the next 64 pieces are on their way while these are walked
            piece_of(base + (int64_t)kAccWaves * kWave + lane, next_len, next_addr);
            // A piece is read as the aligned 16-byte chunks it touches, one chunk per lane and load (four neighbours
            // per lane keep the number of load instructions, and of the LDS additions behind them, at a quarter of
            // what one neighbour per lane costs; a compute unit retires such instructions at a fixed pace whatever
            // number of their lanes is active).  The chunks of the wave's 64 pieces are numbered end to end; which
            // piece a chunk belongs to follows from counting piece starts up to it: the starts inside the current
            // span of chunks are bits in LDS, the pieces' records a small table in LDS indexed by their rank among
            // the nonempty ones.  The entries of a piece's first and last chunk that lie outside the piece (the
            // neighbouring windows' or rows') are masked; an aligned 16-byte read that holds at least one entry of
            // the piece stays inside that entry's page.
            const int64_t lo_byte = A0 + addr * 4, hi_byte = lo_byte + (int64_t)len * 4;
            const int64_t chunk0 = lo_byte & ~(int64_t)15;
            const uint32_t nc = len ? (uint32_t)((hi_byte - 1 - chunk0) >> 4) + 1u : 0u;
            const uint32_t inc = wave_inclusive_scan(nc);
            const uint32_t total = __shfl(inc, kWave - 1, kWave);
            const uint32_t ustart = inc - nc;
            const bool nonempty = nc != 0;
            const uint64_t ne_mask = __ballot(nonempty);
            __builtin_amdgcn_wave_barrier();
            if (nonempty) {
                AccPiece rec;
                rec.origin = chunk0 - (int64_t)ustart * 16; // chunk j of the wave's order starts at origin + 16 j
                rec.lo_rel = (uint32_t)(lo_byte - rec.origin);
                rec.hi_rel = (uint32_t)(hi_byte - rec.origin);
                piece_rec[__popcll(ne_mask & below)] = rec;
            }
            for (uint32_t u0 = 0; u0 < total; u0 += kAccChunks) {
                __builtin_amdgcn_wave_barrier();
                if (lane < 2 * kAccUnroll)
                    starts[lane] = 0;
                __builtin_amdgcn_wave_barrier();
                const uint32_t rel = ustart - u0; // wraps for pieces that start before the span
                if (nonempty && rel < (uint32_t)kAccChunks)
                    atomicOr(starts + (rel >> 5), 1u << (rel & 31u));
                __builtin_amdgcn_wave_barrier();
                int rank = __popcll(__ballot(nonempty && ustart < u0)) - 1; // piece that holds chunk u0 - 1
                uint4 v[kAccUnroll] = {};
                uint32_t keep = 0; // 4 bits per step: which of the 4 entries belong to the piece
#pragma unroll
                for (int u = 0; u < kAccUnroll; ++u) {
                    if (u0 + (uint32_t)(u * kWave) >= total) // (the same for all lanes)
                        break;
                    const uint32_t j = u0 + (uint32_t)(u * kWave + lane);
                    const uint64_t m = reinterpret_cast<const uint64_t *>(starts)[u];
                    const int mine = rank + __popcll(m & below_incl);
                    rank += __popcll(m);
                    v[u] = make_uint4(0, 0, 0, 0);
                    if (j < total) {
                        const AccPiece rec = piece_rec[mine];
                        const uint32_t off = j * 16u; // of the lane's 16 bytes, from origin
                        uint32_t k4 = 0;
#pragma unroll
                        for (uint32_t e = 0; e < 4; ++e)
                            k4 |= (off + 4u * e >= rec.lo_rel && off + 4u * e < rec.hi_rel) ? 1u << e : 0u;
                        v[u] = *reinterpret_cast<const uint4 *>(rec.origin + (int64_t)off);
                        keep |= k4 << (4 * u);
                    }
                }
#pragma unroll
                for (int u = 0; u < kAccUnroll; ++u) {
                    if (u0 + (uint32_t)(u * kWave) >= total)
                        break;
                    const uint32_t xs[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if ((keep >> (4 * u + e)) & 1u) {
                            const uint32_t x = xs[e] - (uint32_t)id0;
                            atomicAdd(&cnt[x >> 1], 1u << ((x & 1u) * 16));
                        }
                }
            }
            len = next_len;
            addr = next_addr;
        }
        first_pieces(slot + G, len, addr);
        __syncthreads();
        // Each wave compacts its part of the window, kWaveWords consecutive words, in one pass: the nonzero counters
        // leave in ascending column order as (column - id0) << 16 | e_v, and are cleared; the wave records where its
        // part went, how many entries it holds and what they weigh.
        const int64_t claimed = (int64_t)claim_s[turn] + (int64_t)wave * room;
        turn ^= 1;
        const int64_t part = blk * kWinParts + wave;
        uint32_t nz = 0;
        uint32_t w32 = 0; // e_v: at most 64 values below 2^16 per lane
        uint64_t w64 = 0; // e_v^2
        if (added_blk) {
            // 16 bytes (8 counters) per lane and access: the lanes' counts of nonzero counters are scanned, every lane
            // writes its own run; a group of 64 such quads without any counter costs one LDS read.  (Packing the
            // nonzero counters of 64 consecutive words by ballots instead, so that a store instruction writes one
            // run of consecutive entries, took four times the steps and more instructions per counter: 9 us
            // against 6 per full window.)
            constexpr int kQuadIts = kWaveWords / 4 / kWave; // quads per lane
            uint4 *mine4 = reinterpret_cast<uint4 *>(cnt + wave * kWaveWords);
            uint32_t *__restrict__ out = a.tmp_ent + claimed;
#pragma unroll
            for (int it = 0; it < kQuadIts; ++it) {
                const uint4 q = mine4[it * kWave + lane];
                const uint32_t xs[4] = {q.x, q.y, q.z, q.w};
                uint32_t c = 0;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    c += ((xs[u] & 0xFFFFu) != 0) + ((xs[u] >> 16) != 0);
                if (__ballot(c != 0) == 0)
                    continue;
                if (c)
                    mine4[it * kWave + lane] = make_uint4(0, 0, 0, 0);
                const uint32_t inc = wave_inclusive_scan_dpp(c);
                uint32_t pos = nz + (inc - c);
                nz += (uint32_t)__builtin_amdgcn_readlane((int)inc, kWave - 1);
                const uint32_t col0 = 2u * (uint32_t)(wave * kWaveWords + 4 * (it * kWave + lane)); // within the window
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t lo = xs[u] & 0xFFFFu, hi = xs[u] >> 16;
                    if (a.squared)
                        w64 += (uint64_t)(lo * lo) + (uint64_t)(hi * hi);
                    else
                        w32 += lo + hi;
                    if (lo)
                        out[pos++] = (col0 + 2 * u) << 16 | lo;
                    if (hi)
                        out[pos++] = (col0 + 2 * u + 1) << 16 | hi;
                }
            }
        }
        const uint64_t wt = wave_sum(a.squared ? w64 : (uint64_t)w32);
        if (lane == 0) {
            a.part_base[part] = claimed;
            a.part_cnt[part] = nz;
            a.part_wt[part] = wt;
        }
        __syncthreads();
    }
}

// one workgroup per minibatch: columns and weight of every window (the sums of its parts), before each of its
// parts, and before each window; columns of the minibatch
__global__ __launch_bounds__(256) void ldw_win_scan_kernel(LwHop a)
{
    __shared__ uint64_t smem[4];
    __shared__ uint64_t carry_c, carry_w;
    const int i = blockIdx.x, tid = threadIdx.x;
    if (a.giveup && *a.giveup) {
        if (tid == 0)
            a.mb_count[i] = 0;
        return;
    }
    if (tid == 0) {
        carry_c = 0;
        carry_w = 0;
    }
    __syncthreads();
    for (int base = 0; base < a.nwin; base += 256) {
        const int w = base + tid;
        const int64_t x = (int64_t)i * a.nwin + w;
        uint64_t c = 0, wt = 0;
        if (w < a.nwin) {
            for (int q = 0; q < kWinParts; ++q) {
                const int64_t part = x * kWinParts + q;
                a.part_off[part] = (uint32_t)c;
                a.part_woff[part] = wt;
                c += a.part_cnt[part];
                wt += a.part_wt[part];
            }
            a.win_cnt[x] = (uint32_t)c;
            a.win_wt[x] = wt;
        }
        uint64_t tc, tw;
        const uint64_t ec = block_exclusive_scan<uint64_t, 256>(c, smem, tc);
        const uint64_t ew = block_exclusive_scan<uint64_t, 256>(wt, smem, tw);
        const uint64_t cc = carry_c, cw = carry_w;
        if (w < a.nwin) {
            a.win_poff[x] = (int64_t)(cc + ec);
            a.win_woff[x] = cw + ew;
        }
        __syncthreads();
        if (tid == 0) {
            carry_c = cc + tc;
            carry_w = cw + tw;
        }
        __syncthreads();
    }
    if (tid == 0)
        a.mb_count[i] = (int64_t)carry_c;
}

// Windows to their place in P, with the inclusive prefix sums of the weights.  A window left the accumulation in
// kWinParts parts (one per wave) whose sizes and weights are on record, so every part has a known place and a
// known weight before it: one wave per part streams it, 64 entries at a time, with lane scans for the sums and
// no workgroup barrier.
constexpr int kPrefixBlock = 16; // entries of P per kept prefix sum
constexpr int kCopyUnroll = 4;
__global__ __launch_bounds__(256) void ldw_p_copy_kernel(LwHop a)
{
    if (a.giveup) {
        if (*a.giveup)
            return;
        if (a.p_off[a.k] > a.p_cap) { // P does not fit what was provided (the same in every workgroup)
            if (blockIdx.x == 0 && threadIdx.x == 0)
                *a.giveup = 1;
            return;
        }
    }
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t nparts = (int64_t)a.k * a.nwin * kWinParts;
    for (int64_t part = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave; part < nparts; part += (int64_t)gridDim.x * 4) {
        const int64_t blk = part / kWinParts;
        const uint32_t cw = a.part_cnt[part];
        if (cw == 0)
            continue;
        const uint32_t o0 = a.part_off[part];
        const int i = (int)(blk / a.nwin);
        const int32_t id0 = (int32_t)(blk % a.nwin) << kWinShift;
        const uint32_t *__restrict__ src = a.tmp_ent + a.part_base[part];
        const int64_t dst = a.p_off[i] + a.win_poff[blk] + o0;
        uint64_t carry = a.win_woff[blk] + a.part_woff[part];
        for (uint32_t x0 = 0; x0 < cw; x0 += kCopyUnroll * kWave) {
            uint32_t ent[kCopyUnroll];
#pragma unroll
            for (int u = 0; u < kCopyUnroll; ++u) {
                const uint32_t x = x0 + u * kWave + lane;
                ent[u] = x < cw ? src[x] : 0u;
            }
#pragma unroll
            for (int u = 0; u < kCopyUnroll; ++u) {
                const uint32_t x = x0 + u * kWave + lane;
                const uint32_t c = ent[u] & 0xFFFFu;
                // e_v < 2^16: sums of 64 weights e_v fit 32 bits; e_v^2 is summed as two 16-bit halves
                uint64_t inc;
                if (a.squared) {
                    const uint32_t wq = c * c;
                    inc = ((uint64_t)wave_inclusive_scan_dpp(wq >> 16) << 16) + wave_inclusive_scan_dpp(wq & 0xFFFFu);
                } else {
                    inc = wave_inclusive_scan_dpp(c);
                }
                if (x < cw) {
                    a.p_col[dst + x] = id0 + (int32_t)(ent[u] >> 16);
                    a.p_cnt[dst + x] = c;
                    // the draws find their block of kPrefixBlock entries of P by these sums and walk the weights
                    // inside it: only the sum at the last entry of every such block (absolute index in P) is kept
                    if (((dst + x) & (kPrefixBlock - 1)) == kPrefixBlock - 1)
                        a.prefix[(dst + x) / kPrefixBlock] = carry + inc;
                }
                carry += __shfl(inc, kWave - 1, kWave);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// SAMPLE: one workgroup per minibatch
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void ldw_draw_kernel(LwHop a)
{
    __shared__ uint32_t key[kMaxWinSampled];
    __shared__ uint32_t smem[16];
    __shared__ uint64_t top[kDrawTop];
    const int i = blockIdx.x, tid = threadIdx.x;
    if (a.giveup && (*a.giveup || a.p_off[a.k] > a.p_cap)) { // no P: the minibatch gets no columns
        if (tid == 0)
            a.mb_count[i] = 0;
        return;
    }
    const int64_t p0 = a.p_off[i], C = a.p_off[i + 1] - p0;
    uint32_t M = 1024; // sorted size: a power of two >= s, at least one slot per thread
    while (M < (uint32_t)a.s)
        M <<= 1;
    // inclusive weight sums are on record at the last entry of every block of kPrefixBlock entries (absolute
    // index in P): blocks B0 .. B0 + nb - 1 end inside this minibatch's row; W = the row sum
    const int64_t B0 = p0 / kPrefixBlock, nb = (p0 + C) / kPrefixBlock - B0;
    const uint64_t *__restrict__ pre = a.prefix + B0;
    const int64_t last_win = (int64_t)i * a.nwin + a.nwin - 1;
    const uint64_t W = a.win_woff[last_win] + a.win_wt[last_win];
    const uint64_t rk = row_key(a.hopkey, a.mb_base + (uint32_t)i, kNoVertex);
    // Every draw searches the recorded sums; probes far apart in memory cost a trip to memory each and follow one
    // another.  The sums at the end of every group of 2^st blocks (at most kDrawTop groups) are copied to LDS
    // first: a draw finds its group there and only the last st probes go to memory, close to one another.
    int st = 0;
    while ((nb >> st) > kDrawTop)
        ++st;
    const int64_t ntop = nb >> st;
    for (int64_t t = tid; t < ntop; t += 1024)
        top[t] = pre[((t + 1) << st) - 1];
    __syncthreads();
    for (uint32_t j = tid; j < M; j += 1024) {
        uint32_t v = kEmptySlot;
        if (j < (uint32_t)a.s && C > 0) { // an empty aggregated neighbourhood samples nothing
            const uint64_t r = bounded64(draw64(rk, j), W);
            int64_t lo = 0, hi = ntop; // first group whose last recorded sum exceeds r (ntop: the blocks after the groups)
            while (lo < hi) {
                const int64_t mid = lo + ((hi - lo) >> 1);
                if (top[mid] > r)
                    hi = mid;
                else
                    lo = mid + 1;
            }
            hi = lo < ntop ? ((lo + 1) << st) - 1 : nb; // first block whose recorded sum exceeds r (nb: the unrecorded tail)
            lo <<= st;
            while (lo < hi) {
                const int64_t mid = lo + ((hi - lo) >> 1);
                if (pre[mid] > r)
                    hi = mid;
                else
                    lo = mid + 1;
            }
            uint64_t acc = lo > 0 ? pre[lo - 1] : 0ull;
            int64_t e = (B0 + lo) * kPrefixBlock;
            if (e < p0)
                e = p0;
            const int64_t end = p0 + C - 1; // the smallest t with prefix[t] > r exists below the row's end: W > r
            for (; e < end; ++e) {
                acc += ldw_weight(a.p_cnt[e], a.squared);
                if (acc > r)
                    break;
            }
            v = (uint32_t)a.p_col[e];
        }
        key[j] = v;
    }
    __syncthreads();
    for (uint32_t size = 2; size <= M; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t t = tid; t < (M >> 1); t += 1024) {
                const uint32_t lo = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                const uint32_t hi = lo | stride;
                const uint32_t x = key[lo], y = key[hi];
                if ((x > y) == ((lo & size) == 0)) {
                    key[lo] = y;
                    key[hi] = x;
                }
            }
            __syncthreads();
        }
    }
    // thread t owns sorted slots [t per, (t+1) per); the first of every run of equal columns stays
    const uint32_t per = M >> 10;
    uint32_t heads = 0;
    for (uint32_t j = tid * per; j < (tid + 1) * per; ++j)
        heads += (key[j] != kEmptySlot && (j == 0 || key[j] != key[j - 1])) ? 1u : 0u;
    uint32_t total;
    uint32_t rank = block_exclusive_scan<uint32_t, 1024>(heads, smem, total);
    int32_t *__restrict__ out = a.sel_tmp + (int64_t)i * a.s;
    for (uint32_t j = tid * per; j < (tid + 1) * per; ++j)
        if (key[j] != kEmptySlot && (j == 0 || key[j] != key[j - 1]))
            out[rank++] = (int32_t)key[j];
    if (tid == 0)
        a.mb_count[i] = total;
}

__global__ __launch_bounds__(256) void ldw_sel_copy_kernel(LwHop a)
{
    if (a.giveup && *a.giveup)
        return;
    const int i = blockIdx.x;
    const int64_t c0 = a.mb_coloff[i], cnt = a.mb_coloff[i + 1] - c0;
    for (int64_t j = threadIdx.x; j < cnt; j += 256)
        a.col_vertex[c0 + j] = a.sel_tmp[(int64_t)i * a.s + j];
}

// ---------------------------------------------------------------------------------------------
// EXTRACT: blockIdx.y = minibatch; the workgroups of a minibatch share its rows wave by wave
// ---------------------------------------------------------------------------------------------
// kFilterBits hash bits: all of them index the filter bitmap (16 KB: with up to 4096 sampled columns about 1.5 % of
// the neighbours pass, half of what a 2^16-bit filter lets through; twice the size would cost the second workgroup
// per compute unit), the low 13 the table
constexpr int kFilterBits = 17;
__device__ inline uint32_t ldw_hash(uint32_t v) { return (v * 0x9E3779B1u) >> (32 - kFilterBits); }
static_assert(kHashSlots == 1 << 13, "hash width out of step");
constexpr int kFilterWords = (1 << kFilterBits) / 32;

__global__ __launch_bounds__(kExtThreads) void ldw_extract_kernel(LwHop a)
{
    __shared__ uint32_t hkey[kHashSlots];
    __shared__ uint16_t hval[kHashSlots];
    __shared__ uint32_t maybe[kFilterWords]; // bit h set: some sampled column hashes to h
    __shared__ uint32_t queue_all[kExtWaves * 2 * kWave]; // per wave: neighbours that passed the filter, in row order
    if (a.giveup && *a.giveup)
        return;
    const int i = blockIdx.y, tid = threadIdx.x, lane = tid & (kWave - 1);
    uint32_t *queue = queue_all + (tid / kWave) * 2 * kWave;
    const int64_t c0 = a.mb_coloff[i];
    const int32_t ns = (int32_t)(a.mb_coloff[i + 1] - c0);
    const int64_t x0 = a.mb_gtileoff[i], ntiles = a.mb_gtileoff[i + 1] - x0;
    if (ns == 0 || (int64_t)blockIdx.x * kExtWaves >= ntiles)
        return; // nothing sampled: every row stays empty (the counters start at zero)
    for (int x = tid; x < kHashSlots; x += kExtThreads)
        hkey[x] = kEmptySlot;
    for (int x = tid; x < kFilterWords; x += kExtThreads)
        maybe[x] = 0;
    __syncthreads();
    for (int j = tid; j < ns; j += kExtThreads) {
        const uint32_t v = (uint32_t)a.col_vertex[c0 + j];
        atomicOr(&maybe[ldw_hash(v) >> 5], 1u << (ldw_hash(v) & 31u));
        uint32_t slot = ldw_hash(v) & (kHashSlots - 1);
        while (atomicCAS(&hkey[slot], kEmptySlot, v) != kEmptySlot)
            slot = (slot + 1) & (kHashSlots - 1);
        hval[slot] = (uint16_t)j;
    }
    __syncthreads();
    const uint64_t below = (1ull << lane) - 1ull;
    unsigned long long *rowcnt = reinterpret_cast<unsigned long long *>(a.out_rowptr);
    const int64_t nrows = a.mb_rowoff[a.k];
    // tiles cost very different amounts (one long piece, or many short rows): the minibatch's tiles go to
    // whichever of its waves is free, off a shared counter, until none is left
    // A wave's first tile is its own number among the minibatch's waves; the counter hands out the tiles after
    // those.  The next tile is asked for before the current one is worked on, so that the answer (a trip to the
    // counter's home in memory, shared by all waves of the minibatch) is there when it is needed.
    const int64_t nwaves = (int64_t)gridDim.x * kExtWaves;
    int64_t t = (int64_t)blockIdx.x * kExtWaves + tid / kWave;
    while (t < ntiles) {
        int64_t t_next = 0;
        if (lane == 0)
            t_next = nwaves + (int64_t)atomicAdd(a.tile_queue + i, 1ull);
        const int64_t g0 = a.mb_goff[i] + t * a.tile;
        const int64_t g1 = min(g0 + a.tile, a.mb_goff[i + 1]);
        ldw_walk_tile(a, g0, g1, a.tile_row[x0 + t], nrows,
                      [&](int64_t r, int64_t rs, int64_t re, int64_t shift, int64_t g, int64_t pe) {
            (void)re;
            int32_t *__restrict__ out = a.xtmp + g; // the kept neighbours of a piece start where the piece starts
            uint32_t kept = 0;
            uint32_t qn = 0; // neighbours waiting in the wave's queue (the same in every lane)
            // looks the first n <= 64 queued neighbours up in the table, appends the local columns of those found
            // to the piece's output in queue order, and moves the rest of the queue down
            auto drain = [&](uint32_t n) {
                __builtin_amdgcn_wave_barrier();
                const uint32_t val = (uint32_t)lane < n ? queue[lane] : kEmptySlot;
                int32_t local = -1;
                if (val != kEmptySlot) {
                    uint32_t slot = ldw_hash(val) & (kHashSlots - 1);
                    uint32_t kx;
                    while ((kx = hkey[slot]) != kEmptySlot) {
                        if (kx == val) {
                            local = hval[slot];
                            break;
                        }
                        slot = (slot + 1) & (kHashSlots - 1);
                    }
                }
                const uint64_t found = __ballot(local >= 0);
                if (local >= 0)
                    out[kept + __popcll(found & below)] = local;
                kept += __popcll(found);
                const uint32_t rest = qn - n;
                const uint32_t moved = (uint32_t)lane < rest ? queue[kWave + lane] : 0u;
                __builtin_amdgcn_wave_barrier();
                if ((uint32_t)lane < rest)
                    queue[lane] = moved;
                qn = rest;
                __builtin_amdgcn_wave_barrier();
            };
            for (int64_t p0 = g; p0 < pe; p0 += kStreamUnroll * kWave) {
                const int32_t *__restrict__ from = a.A_col + (shift + p0); // slot x of the step is position p0 + x
                const int32_t nslots = (int32_t)min<int64_t>(pe - p0, kStreamUnroll * kWave);
                uint32_t v[kStreamUnroll];
#pragma unroll
                for (int u = 0; u < kStreamUnroll; ++u) {
                    const int32_t x = u * kWave + lane;
                    v[u] = x < nslots ? (uint32_t)from[x] : kEmptySlot;
                }
                // almost no neighbour is a sampled column: one bit per hash value answers "certainly not" for
                // nearly all of them with a single LDS read each (all of a step's reads in flight together).
                // The few that pass are queued in row order; the table is searched a full wave of them at a
                // time (and at the end of the piece), not step by step
                uint32_t word[kStreamUnroll];
#pragma unroll
                for (int u = 0; u < kStreamUnroll; ++u)
                    word[u] = maybe[ldw_hash(v[u]) >> 5];
#pragma unroll
                for (int u = 0; u < kStreamUnroll; ++u) {
                    const bool pass = v[u] != kEmptySlot && ((word[u] >> (ldw_hash(v[u]) & 31u)) & 1u);
                    const uint64_t pm = __ballot(pass);
                    if (pm == 0)
                        continue;
                    if (pass)
                        queue[qn + __popcll(pm & below)] = v[u];
                    qn += __popcll(pm);
                    if (qn >= (uint32_t)kWave)
                        drain(kWave);
                }
            }
            while (qn)
                drain(qn < (uint32_t)kWave ? qn : (uint32_t)kWave);
            if (lane == 0) {
                if (g == rs)
                    a.first_cnt[r] = kept; // the piece a row starts with
                else
                    a.tile_cnt[x0 + t] = kept; // the piece a tile starts with, of a row begun earlier
                if (kept)
                    atomicAdd(&rowcnt[r], (unsigned long long)kept);
            }
        });
        t = __shfl(t_next, 0, kWave);
    }
}

// rows to their place, piece by piece: 16 lanes per row
__global__ __launch_bounds__(256) void ldw_extract_copy_kernel(LwHop a)
{
    const int64_t R = a.mb_rowoff[a.k];
    if (a.giveup) {
        if (*a.giveup)
            return;
        if (a.out_rowptr[R] > a.col_cap) { // the kept neighbours do not fit what was provided
            if (blockIdx.x == 0 && threadIdx.x == 0)
                *a.giveup = 1;
            return;
        }
    }
    const int sub = threadIdx.x & 15;
    const int64_t groups = (int64_t)gridDim.x * 16;
    for (int64_t r = (int64_t)blockIdx.x * 16 + threadIdx.x / 16; r < R; r += groups) {
        int64_t o = a.out_rowptr[r];
        const int64_t total = a.out_rowptr[r + 1] - o;
        if (total == 0)
            continue;
        const int i = a.row_mb[r];
        const int64_t rs = a.gather_off[r], re = a.gather_off[r + 1];
        const int64_t gm = a.mb_goff[i], xm = a.mb_gtileoff[i];
        int64_t g = rs;
        int64_t cnt = a.first_cnt[r];
        int64_t t = (rs - gm) / a.tile;
        while (true) {
            for (int64_t j = sub; j < cnt; j += 16)
                a.out_col[o + j] = a.xtmp[g + j];
            o += cnt;
            ++t;
            g = gm + t * a.tile;
            if (g >= re)
                break;
            cnt = a.tile_cnt[xm + t];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------
size_t ldw_accumulate_lds_bytes()
{
    return (size_t)(kWinWords + 3 * kAccWaves + 4) * sizeof(uint32_t) + (size_t)kAccWaves * (kWave + kAccUnroll / 2) * sizeof(AccPiece);
}

static void launch_ldw_tiles(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_plan_kernel, dim3(1), dim3(1024), 0, L.stream, a);
    hipLaunchKernelGGL(ldw_tile_rows_kernel, dim3(grid_for(L, (a.tiles_bound + 255) / 256, 8)), dim3(256), 0, L.stream, a);
}

void launch_ldw_bounds(const Launch &L, const LwHop &a)
{
    launch_ldw_tiles(L, a);
    if (!a.index)
        hipLaunchKernelGGL(ldw_bounds_kernel, dim3(grid_for(L, (a.tiles_bound + 3) / 4, 8)), dim3(256), 0, L.stream, a);
    const int64_t ttiles = ((a.nwin + 1 + 63) / 64) * ((a.rows_bound + 63) / 64);
    hipLaunchKernelGGL(ldw_bounds_transpose_kernel, dim3(grid_for(L, ttiles, 8)), dim3(256), 0, L.stream, a);
}

void launch_ldw_index(const Launch &L, const LwHop &a)
{
    launch_ldw_tiles(L, a);
    hipLaunchKernelGGL(ldw_bounds_kernel, dim3(grid_for(L, (a.tiles_bound + 3) / 4, 8)), dim3(256), 0, L.stream, a);
}

int launch_ldw_accumulate(const Launch &L, const LwHop &a)
{
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(ldw_accumulate_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)ldw_accumulate_lds_bytes()) != hipSuccess)
            (void)hipGetLastError(); // not required on every runtime; the launch below reports real failures
        attr_set = true;
    }
    hipLaunchKernelGGL(ldw_win_added_kernel, dim3(grid_for(L, (int64_t)a.k * a.nwin, 8)), dim3(256), 0, L.stream, a);
    hipLaunchKernelGGL(ldw_accumulate_kernel, dim3(grid_for(L, (int64_t)a.k * a.nwin, 1)), dim3(kAccThreads),
                       ldw_accumulate_lds_bytes(), L.stream, a);
    if (hipGetLastError() != hipSuccess)
        return -1;
    hipLaunchKernelGGL(ldw_win_scan_kernel, dim3(a.k), dim3(256), 0, L.stream, a);
    return 0;
}

void launch_ldw_p_copy(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_p_copy_kernel, dim3(grid_for(L, ((int64_t)a.k * a.nwin * kWinParts + 3) / 4, 8)), dim3(256), 0, L.stream, a);
}

void launch_ldw_draw(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_draw_kernel, dim3(a.k), dim3(1024), 0, L.stream, a);
}

void launch_ldw_sel_copy(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_sel_copy_kernel, dim3(a.k), dim3(256), 0, L.stream, a);
}

void launch_ldw_extract(const Launch &L, const LwHop &a)
{
    int64_t per_mb = (L.num_cu * 2 + a.k - 1) / a.k; // workgroups per minibatch: about 2 per compute unit in all
    per_mb = std::min<int64_t>(per_mb, (a.tiles_bound + kExtWaves - 1) / kExtWaves); // never more than there are tiles
    per_mb = std::max<int64_t>(per_mb, 1);
    hipLaunchKernelGGL(ldw_extract_kernel, dim3((unsigned)per_mb, a.k), dim3(kExtThreads), 0, L.stream, a);
}

void launch_ldw_extract_copy(const Launch &L, const LwHop &a)
{
    hipLaunchKernelGGL(ldw_extract_copy_kernel, dim3(grid_for(L, (a.rows_bound + 15) / 16, 8)), dim3(256), 0, L.stream, a);
}

} // namespace bms
