// Host-side declarations shared by the translation units of libbms.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <functional>

namespace bms {

// Per-minibatch vertex set over [0,n): a bitmap in 64-byte lines plus, per line, the number of
// set bits before it (the rank of the line's first vertex).  It serves as the dedup structure
// ("remove empty columns", Sec. 4.1.3), as the ordered compaction that yields the next frontier,
// and as the membership/rank lookup of column extraction (Sec. 4.2.3).
// Invariant between calls: every word is zero.
struct VSet {
    uint32_t *words = nullptr;       // k * nw
    uint32_t *line_prefix = nullptr; // k * nl
    int64_t *chunk_off = nullptr;    // k * nc : set bits per chunk, then their exclusive scan
    int64_t nw = 0, nl = 0;
    int32_t nc = 0;
};

struct Launch {
    hipStream_t stream;
    int num_cu;
    int64_t *scan_tmp = nullptr; // scratch for scans that span several workgroups: one value per 4096 inputs
    int64_t scan_tmp_len = 0;
};

int grid_for(const Launch &L, int64_t blocks, int per_cu);
// called by multi-kernel launchers before each kernel (group) so that it can be timed on its own
using StageMark = std::function<void(const char *)>;

// ---- common ----
void launch_csr_check(const Launch &, const int64_t *rowptr, const int32_t *col, int64_t n, int64_t nnz,
                      int32_t *flag /*device, zeroed*/, unsigned long long *maxdeg /*device, zeroed*/);
void launch_validate_seeds(const Launch &, const int32_t *seeds, int32_t k, int32_t b, int64_t n, const VSet &,
                           int32_t *flag);
void launch_clear_seed_bits(const Launch &, const int32_t *seeds, int32_t k, int32_t b, int64_t n, const VSet &);
void launch_iota_offsets(const Launch &, int64_t *off, int32_t k, int64_t step); // off[i] = i*step, i<=k
// max_out (optional): receives the largest number of tiles any segment has
void launch_plan_tiles(const Launch &, const int64_t *seg_off, int32_t k, int32_t tile, int64_t *seg_tileoff,
                       int64_t *max_out = nullptr);
void launch_plan_tiles3(const Launch &, const int64_t *seg_off, int32_t k, int32_t tile0, int64_t *off0, int32_t tile1,
                        int64_t *off1, int32_t tile2, int64_t *off2);
// exclusive scan of vals[0..*count) in place, vals[*count] = total; total also stored to *total_out and,
// when tail_ptr != nullptr, to tail_ptr[*tail_idx].  count_bound = host-side upper bound of *count (0: unknown);
// long arrays are scanned by many workgroups when the launch context carries scratch for it
void launch_scan_i64(const Launch &, int64_t *vals, const int64_t *count, int64_t *total_out, int64_t *tail_ptr,
                     const int64_t *tail_idx, int64_t count_bound = 0);
void launch_vset_rank(const Launch &, const VSet &, int32_t k, int64_t *mb_coloff /*k+1*/, int32_t *col_vertex,
                      int64_t *ncols_out);
void launch_vset_clear(const Launch &, const VSet &, int32_t k, const int64_t *mb_coloff, const int32_t *col_vertex,
                       int64_t ncols_bound);

// ---- node-wise ----
struct NwHop {
    const int64_t *A_rowptr;
    const int32_t *A_col;
    int64_t n;
    int32_t k;
    int32_t s;
    uint64_t hopkey;
    uint32_t mb_base;
    const int32_t *row_vertex; // stacked frontier
    const int64_t *mb_rowoff;  // k+1
    int64_t *mb_tileoff;       // k+1
    int64_t *row_beg;          // scratch, rows
    int32_t *row_deg;          // scratch, rows
    int64_t *tile_off;         // scratch, tiles+1
    int64_t *out_rowptr;       // rows+1
    int32_t *out_col;          // nnz
    int64_t *nnz_out;          // device scalar
    int64_t rows_bound;        // host-side upper bound of the row count
    int32_t max_degree;
    int32_t self_entry;        // 1: every row carries its own vertex as one more entry after the sampled ones
    int32_t replace;           // 1: the s draws of a row are independent, the row keeps the distinct picks
    int32_t *row_cnt;          // scratch, rows: distinct picks per row (only with replace and s > 32)
    // EXTRACT's count of sampled ids per (minibatch, id-range segment), taken while the ids are staged in LDS
    // (nullptr: not wanted); the caller has zeroed the counters
    uint32_t *seg_cnt;         // k * seg_C
    int32_t seg_C, seg_shift;  // segment of an id = id >> seg_shift, < seg_C <= kMaxFusedSegments
    const uint16_t *seg_tab;   // not nullptr: segment of an id = seg_tab[id >> seg_shift] (kMaxCells + 1 entries at most)
};
constexpr int kMaxFusedSegments = 512;
void launch_nw_rows(const Launch &, const NwHop &);
// set_bits: also mark every sampled vertex in the minibatch's vertex set (bitmap EXTRACT path).
// Returns true when the kernel also took the per-segment counts asked for in NwHop::seg_cnt (it can when every
// workgroup stays with one minibatch: one row per lane, no more minibatches than workgroups).
bool launch_nw_sample(const Launch &, const NwHop &, const VSet &, bool set_bits);
void launch_nw_relabel(const Launch &, const NwHop &, const VSet &);
// rows that carry a trailing entry for their own vertex -> the CSR without it + that entry per row;
// *rows = number of rows (device), *nnz_slot: entries on input, entries - rows on output
void launch_nw_strip_self(const Launch &, const int64_t *rowptr_in, const int32_t *col_in, const int64_t *rows,
                          int64_t rows_bound, int64_t *rowptr_out, int32_t *col_out, int32_t *row_self,
                          int64_t *nnz_slot);

// EXTRACT ("remove empty columns", Sec. 4.1.3).  Main path: the sampled ids of every minibatch are cut into C
// id-range segments, the segments are ranked in LDS, and the ranks travel back to the entries' positions through the
// run structure of the cut (kernels_dedup_sort.hip).  Fallback for crowded id ranges and path of small hops: one
// workgroup per minibatch over id-range bins (kernels_dedup.hip).
constexpr int kBucketBits = 15;     // ids per bucket = 2^15 (a 4 KB bitmap per wave in LDS)
constexpr int kMaxBuckets = 8000;   // two uint32 per bucket must fit beside 16 wave bitmaps in 160 KB of LDS
struct DedupArgs {
    int32_t k;
    int32_t nbuckets;    // ceil(n / 2^kBucketBits) <= kMaxBuckets
    int64_t *mb_edgeoff; // k+1, scratch
    int32_t *col;        // in: sampled global ids (stacked), out: local column indices
    uint64_t *pairs;     // nnz, scratch (bin path): (id << 32 | position in minibatch) partitioned by bin, then (bin, rank, position)
    uint64_t *utmp;      // nnz, scratch (bin path): (bin, rank, id) of every distinct id, at its group's slots
    uint32_t *bin_base;  // k * stride, scratch: distinct ids of the minibatch before each bin's group / each segment
    uint64_t *back;      // nnz, scratch (bin path): (local column << 32 | position) grouped by destination range
    int64_t *split_tileoff, *place_tileoff; // k+1 each, scratch (bin path)
    uint32_t *place_cursor;                 // one per destination range, scratch (bin path)
    int64_t *mb_count;   // k, scratch: distinct ids per minibatch
    int32_t stride;      // entries of bin_base per minibatch (>= nbuckets and >= C)
    // segment path (C == 0: not used)
    int32_t C;           // id-range segments per minibatch = ceil(n / 2^cshift) <= kMaxSegments
    int32_t cshift;      // segment of an id = id >> cshift
    int32_t by_bitmap;   // 1: every segment is ranked through a bitmap of its id range (dense hops); 0: by counting
    // Segments of unequal width (ids that crowd parts of [0, n), e.g. ids sorted by degree): cells of 2^fshift ids,
    // tab[id >> fshift] = segment of the cell, seg_first[c] = first cell of segment c (C + 1 entries; segments
    // past the last one in use are empty).  tab == nullptr: every segment is 2^cshift ids wide.
    const uint16_t *tab;
    const uint32_t *seg_first;
    int32_t fshift;
    int32_t wbits_max;   // log2 of the ids the bitmap kernel's LDS holds: no segment it is given is wider
    uint32_t *seg_cnt;   // k * C: entries per segment, later distinct ids per segment
    uint32_t *seg_off;   // k * (C+1): exclusive scan of the entry counts
    uint32_t *seg_cursor; // k * C
    int64_t *big_tileoff; // k+1: tiles of kCutTile positions
    uint32_t *big_list;  // k * C: segments that one workgroup of the ranking kernel does not take (too many entries, or
                         // too many of them in one narrow id range): ranked through a bitmap of the id range
    uint32_t *big_count; // device counter of big_list (the word after `fallback`)
    int32_t *fallback;   // device flag: a segment fits neither ranking kernel, the per-minibatch kernel takes the hop
    uint32_t *ids_seg;   // nnz: the sampled ids grouped by segment (minibatch i, segment c at mb_edgeoff[i] + seg_off[c])
    uint32_t *loc;       // nnz, by position: segment << 14 | place inside the run its tile appended to that segment
    uint32_t *run_gpos;  // tiles * C: where the run of (tile, segment) starts inside the minibatch's part of ids_seg
    uint32_t *run_cnt;   // tiles * C: its length
    uint16_t *ranks;     // nnz, parallel to ids_seg: rank of the id among the distinct ids of its segment
    uint32_t *uids;      // nnz: the distinct ids of a segment in ascending order, at the head of the segment's slots
};
constexpr int kCutTile = 8192; // positions per tile of the count, split and un-split kernels
constexpr int kSegCap = 65535;      // most entries a segment may hold: the rank of an id inside its segment has 16 bits
constexpr int kMaxSegments = 2560;  // 3 words each beside the staging of the split / un-split kernels must fit in 160 KB of LDS
constexpr int kMaxCells = 4096;      // cells of the table that maps ids to segments of unequal width
constexpr int kMaxBitmapShift = 20; // the bitmap ranking kernel holds 2^cshift bits in LDS (128 KB)
// EXTRACT of a hop by id-range segments (C > 0).  counted: the per-segment counts are there already.  Also writes
// the next hop's row tiles (next_tileoff, k + 2 entries as launch_plan_tiles with max_out gives them).  `done` is a
// device word that is zero between launches.
void launch_nw_extract_segments(const Launch &, const DedupArgs &, const int64_t *out_rowptr, const int64_t *mb_rowoff,
                                int64_t *mb_coloff, int32_t *col_vertex, int64_t *ncols_out, int64_t *next_tileoff,
                                uint32_t *done, int64_t nnz, bool counted, const StageMark &mark);
void launch_nw_dedup_unsplit(const Launch &, const DedupArgs &, int64_t nnz);
// Builds the table of segments of unequal width for a hop from a sample of its staged ids: tab (cells + 1 entries),
// seg_first (C + 1), at most C segments, each holding about target_per_mb ids of a minibatch and at most
// 2^max_wbits ids wide (max_wbits >= 32: any width).  hist: scratch of kMaxCells + 1 words.
void launch_nw_dedup_table(const Launch &, const int32_t *col, const int64_t *nnz, int64_t nnz_bound, int64_t n, int32_t k,
                           int32_t fshift, int32_t C, int32_t target_per_mb, int32_t max_wbits, uint32_t *hist,
                           uint16_t *tab, uint32_t *seg_first);
void launch_nw_dedup_front(const Launch &, const DedupArgs &, const int64_t *mb_coloff, int32_t *col_vertex, int64_t nnz);
// EXTRACT of a hop by the per-minibatch kernel (C == 0); returns 0, or -1 when the launch was refused
int launch_nw_dedup_bucket(const Launch &, const DedupArgs &, const int64_t *out_rowptr, const int64_t *mb_rowoff,
                           int64_t *mb_coloff, int32_t *col_vertex, int64_t *ncols_out, int64_t nnz, const StageMark &mark);
constexpr int kDedupPlaceTile = 8192; // must equal kPlaceTile in kernels_dedup.hip (sizes the cursor array)
constexpr int kDedupSplitTile = 2048; // must equal kSplitTile in kernels_dedup.hip
// mb_edgeoff[i] = rowptr[mb_rowoff[i]], i <= k: first entry of every minibatch in the stacked column array
void launch_mb_edge_offsets(hipStream_t stream, const int64_t *rowptr, const int64_t *mb_rowoff, int32_t k,
                            int64_t *mb_edgeoff);
void launch_offsets_from_counts(const Launch &, const int64_t *mb_count, int32_t k, int64_t *mb_off,
                                int64_t *total_out);
// seed check without a vertex set: range test + per-minibatch sort in LDS (b <= kMaxSortedSeeds)
constexpr int32_t kMaxSortedSeeds = 8192;
void launch_validate_seeds_sorted(const Launch &, const int32_t *seeds, int32_t k, int32_t b, int64_t n, int32_t *flag);
constexpr int32_t kMaxSampledFanout = 2048; // largest fanout that may be smaller than a row's degree

// ---- LADIES ----
constexpr int kGatherTile = 4096; // gathered neighbours handled by one workgroup iteration (16 per lane)
constexpr int kPChunk = 4096;     // dense counters compacted by one workgroup (16 per lane)
constexpr int kPTile = 1024;      // entries of P per prefix-sum tile

struct LdHop {
    const int64_t *A_rowptr;
    const int32_t *A_col;
    int64_t n;
    int32_t k;
    int32_t s;
    int squared;
    uint64_t hopkey;
    uint32_t mb_base;
    const int32_t *row_vertex; // stacked frontier
    const int64_t *mb_rowoff;  // k+1
    int64_t rows_bound;
    // scratch
    int64_t *row_beg;      // rows
    int64_t *gather_off;   // rows+1 : exclusive scan of the frontier's degrees (the gathered order)
    int32_t *row_mb;       // rows   : minibatch of each stacked row
    int64_t *gather_tiles; // device scalar: ceil(D / kGatherTile)
    uint32_t *counters;    // k * n  : dense e_v, all zero between hops
    int64_t *p_chunks;     // k * nchunk + k
    int32_t nchunk;        // ceil(n / kPChunk)
    int64_t *tile_off;     // gather tiles + 1
    // P (result buffers) and its prefix sums
    int64_t *p_off;        // k+1
    int32_t *p_col;
    uint32_t *p_cnt;
    int64_t *p_tileoff;    // k+1
    uint64_t *p_tilesum;   // P tiles
    uint64_t *prefix;      // pnnz, inclusive, restarts per minibatch
    int64_t pnnz_bound;
    // output
    int64_t *out_rowptr;   // rows+1
    int32_t *out_col;
};
void launch_ld_rows(const Launch &, const LdHop &, int64_t *gather_total_out);
void launch_ld_accumulate(const Launch &, const LdHop &);
void launch_ld_p_count(const Launch &, const LdHop &, int64_t *pnnz_out);
void launch_ld_p_fill(const Launch &, const LdHop &);
void launch_ld_prefix(const Launch &, const LdHop &);
void launch_ld_draw(const Launch &, const LdHop &, const VSet &);
void launch_ld_clear_counters(const Launch &, const LdHop &);
void launch_ld_extract_count(const Launch &, const LdHop &, const VSet &, int64_t *nnz_out);
void launch_ld_extract_fill(const Launch &, const LdHop &, const VSet &);
void launch_chunk_scan(const Launch &, int64_t *chunk_off, int32_t k, int32_t nc, int64_t *mb_off, int64_t *total_out);

// ---- LADIES with the column counts accumulated in LDS, window by window ----
constexpr int kWinShift = 16;            // a window = 2^16 vertex ids = 2^16 16-bit counters = 128 KB of LDS
constexpr int kWinParts = 16;            // a window leaves the accumulation in this many parts of equal id range
constexpr int32_t kMaxWinRows = 65535;   // frontier rows per minibatch (a 16-bit counter cannot overflow)
constexpr int32_t kMaxWinSampled = 4096; // columns sampled per minibatch (sorted, then hashed, in LDS)
constexpr int kLwTileMax = 4096;         // positions of the gathered order streamed by one wave at a time: at most
constexpr int kLwTileMin = 1024;         // ... and at least (hops that gather little use small tiles to fill the chip)
struct LwHop {
    const int64_t *A_rowptr;
    const int32_t *A_col;
    int64_t n;
    int32_t k;
    int32_t s;
    int squared;
    uint64_t hopkey;
    uint32_t mb_base;
    const int32_t *row_vertex; // stacked frontier
    const int64_t *mb_rowoff;  // k+1
    int64_t rows_bound;
    const int64_t *row_beg;    // rows   (from launch_ld_rows)
    const int64_t *gather_off; // rows+1 (from launch_ld_rows)
    const int32_t *row_mb;     // rows   (from launch_ld_rows)
    int64_t *mb_goff;          // k+1: gathered position where each minibatch starts
    int64_t *mb_gtileoff;      // k+1: tiles before each minibatch
    int64_t *tile_row;         // tiles: row holding the tile's first position
    uint32_t *tile_cnt;        // tiles: neighbours kept from the piece the tile starts with (row begun earlier)
    uint32_t *first_cnt;       // rows: neighbours kept from the piece the row starts with
    int64_t tiles_bound;       // host-side upper bound of the number of tiles
    int32_t tile;              // positions per tile of this hop (power of two in [kLwTileMin, kLwTileMax])
    unsigned long long *tile_queue; // k+1 counters, zeroed per hop: next tile of each minibatch (extraction), of the hop (boundaries)
    int32_t nwin;              // ceil(n / 2^kWinShift)
    uint32_t *bounds;          // rows_bound * (nwin+1), one list per row
    const uint32_t *index;     // n * (nwin+1): the list of every vertex's whole row, built once per graph; or null
    uint32_t *bounds_t;        // (nwin+1) * rows_bound, the same window-major
    uint32_t *win_added;       // k * nwin: neighbours of the minibatch's rows inside the window
    uint32_t *win_cnt;         // k * nwin: columns of P inside the window
    uint64_t *win_wt;          // k * nwin: their weight
    int64_t *win_poff;         // k * nwin: columns of the minibatch before the window
    uint64_t *win_woff;        // k * nwin: weight of the minibatch before the window
    int64_t *part_base;        // k * nwin * kWinParts: where the part's entries start in tmp_ent
    uint32_t *part_cnt;        // k * nwin * kWinParts: columns of P in the part
    uint64_t *part_wt;         // k * nwin * kWinParts: their weight
    uint32_t *part_off;        // k * nwin * kWinParts: columns of the window before the part
    uint64_t *part_woff;       // k * nwin * kWinParts: their weight
    unsigned long long *cursor; // device scalar: entries of tmp_* in use
    uint32_t *tmp_ent;         // entries of P, part by part: (column - the window's first id) << 16 | e_v
    int64_t *mb_count;         // k
    int64_t *p_off;            // k+1
    int32_t *p_col;
    uint32_t *p_cnt;
    uint64_t *prefix;          // pnnz, inclusive, restarts per minibatch
    int32_t *sel_tmp;          // k * s
    int64_t *mb_coloff;        // k+1
    int32_t *col_vertex;
    int32_t *xtmp;             // D entries: the kept neighbours of row r start at gather_off[r]
    // A call that sizes its buffers from what an earlier call of the same shape needed (no read-back of sizes on the
    // way) runs every kernel behind a flag: the kernel that first sees a size beyond what was provided raises it,
    // every kernel returns at once when it is up (the hop's minibatches then get no columns, so later hops have no
    // rows), and the host repeats the call with read-backs.
    int32_t *giveup;           // device flag, zero when the call starts
    int64_t gathered_cap;      // gathered neighbours D that xtmp, the tiles and the staging array hold
    int64_t p_cap, col_cap;    // entries that p_col / p_cnt, and out_col, hold
    int64_t *out_rowptr;       // rows+1
    int32_t *out_col;
};
void launch_ldw_bounds(const Launch &, const LwHop &); // with an index: the rows' lists are copied from it
void launch_ldw_index(const Launch &, const LwHop &);  // boundary lists of the rows of a hop that is the whole graph
int launch_ldw_accumulate(const Launch &, const LwHop &); // also scans the windows; -1: launch refused
void launch_ldw_p_copy(const Launch &, const LwHop &);
void launch_ldw_draw(const Launch &, const LwHop &);
void launch_ldw_sel_copy(const Launch &, const LwHop &);
void launch_ldw_extract(const Launch &, const LwHop &);
void launch_ldw_extract_copy(const Launch &, const LwHop &);

// ---- feature fetching ----
// out[j, :] = H[ids[j], :]; *flag (device-visible, zeroed by the caller) is set when an id lies outside [0, n)
void launch_feature_fetch(const Launch &, const float *H, int64_t n, int32_t f, const int32_t *ids, int64_t m,
                          float *out, int32_t *flag);

// ---- forward aggregation of one hop ----
struct AggArgs {
    int64_t rows;
    int32_t k;
    int32_t f;
    int mean;
    const int64_t *mb_rowoff; // k+1
    const int64_t *rowptr;    // rows+1
    const int32_t *col;       // local columns
    const int64_t *mb_coloff; // k+1
    const float *X;           // ncols x f
    float *out;               // rows x f
};
void launch_aggregate(const Launch &, const AggArgs &);

} // namespace bms
