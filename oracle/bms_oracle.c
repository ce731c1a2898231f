/*
 * bms_oracle.c -- plain CPU oracle for the matrix-based bulk minibatch sampler.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement
 * of what the sampler computes.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table or
 * helper with the HIP library; the two sides only agree on the written definition
 * of the counter-based random stream and of the selection rules below.
 *
 * What it follows (paper = arxiv 2311.02909):
 *   - Alg. 1 (sampling framework): for each layer  P <- Q A ; P <- NORM(P) ;
 *     Q' <- SAMPLE(P, b, s) ; A^l <- EXTRACT(A, Q, Q').
 *   - Sec. 4.1 (GraphSAGE): Q has one nonzero per row (column = the row's vertex),
 *     so row r of P is the neighbour list of that vertex with equal weights;
 *     SAMPLE picks s distinct nonzeros per row by inverse-transform sampling;
 *     EXTRACT removes the empty columns of Q'.
 *   - Sec. 4.2 (LADIES): Q has one row per minibatch with a nonzero per frontier
 *     vertex, so P's row holds e_v = number of frontier vertices adjacent to v;
 *     SAMPLE draws s columns by inverse-transform sampling; EXTRACT keeps the
 *     frontier's rows of A (Q_R A) and the sampled columns ((Q_R A) Q_C).
 *   - Eq. 1 (bulk sampling): the k minibatches are stacked vertically; every
 *     minibatch is processed independently, so stacking is concatenation.
 *
 * Readings this oracle fixes where the paper leaves a choice (all integer, so
 * that exactly one output is correct):
 *   - NORM is kept implicit: weights stay integers (1 per neighbour for
 *     GraphSAGE, e_v -- or e_v^2 with the `squared` flag, the form of the
 *     definition in Sec. 2.2 -- for LADIES) and a draw is an integer in [0, W),
 *     W = row sum.  Dividing by W and drawing in [0,1) selects the same column.
 *   - ITS picks the smallest t whose inclusive prefix sum exceeds the draw.
 *   - GraphSAGE "without replacement": draw j is made on the weight vector with
 *     the j already chosen entries set to zero (W = deg - j).  Rows with
 *     deg <= s keep every neighbour.
 *   - LADIES: s draws with replacement from the one row, then duplicates removed.
 *   - EXTRACT orders the surviving columns by ascending vertex id; that list is
 *     the next layer's frontier (no union with the current frontier).
 *   - Two GraphSAGE variants, off by default: ORC_UNION_DST keeps the current
 *     frontier's vertices as columns too (next frontier = frontier + sampled
 *     vertices, the convention of samplers whose layers also use a vertex's own
 *     features) and reports each row's own column; ORC_REPLACE makes the s draws
 *     of a row independent (ITS with replacement: the repeat-until-distinct step
 *     of Sec. 4.1.2 left out) and keeps the distinct picks.
 *   - Random stream: stateless counter hash of (seed, hop, minibatch, vertex,
 *     draw index), defined by orc_rowkey / orc_draw32 / orc_draw64 below.
 *
 * Parity pins for every function here live in tests/ (brute force with dense
 * matrices, closed forms, the paper's worked LADIES example, chi-square).
 * Unpinned: nothing computed here; what is unpinned is the effect of these
 * samples on training accuracy, which is outside this build.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Counter-based random stream                                         */
/* ------------------------------------------------------------------ */

#define ORC_GOLD64 0x9E3779B97F4A7C15ULL /* floor(2^64 / golden ratio), odd */
#define ORC_GOLD32 0x9E3779B9U           /* floor(2^32 / golden ratio), odd */
#define ORC_NOVERTEX 0xFFFFFFFFU         /* vertex field of a LADIES key    */

/* 64-bit finaliser: the output function of the SplitMix64 generator. */
uint64_t orc_mix64(uint64_t x)
{
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

/* 32-bit finaliser: two xorshift-multiply rounds (bijective on uint32). */
uint32_t orc_fin32(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7FEB352DU;
    x ^= x >> 15;
    x *= 0x846CA68BU;
    x ^= x >> 16;
    return x;
}

/* Key of one distribution: (seed, hop) first, then (minibatch, vertex). */
uint64_t orc_rowkey(uint64_t seed, int32_t hop, uint32_t mb, uint32_t vertex)
{
    uint64_t hopkey = orc_mix64(seed ^ (ORC_GOLD64 * (uint64_t)(hop + 1)));
    return orc_mix64(hopkey ^ (((uint64_t)mb << 32) | (uint64_t)vertex));
}

/* j-th 32-bit random number of a distribution. */
uint32_t orc_draw32(uint64_t key, uint32_t j)
{
    uint32_t lo = (uint32_t)key, hi = (uint32_t)(key >> 32);
    return orc_fin32(orc_fin32(lo + j * ORC_GOLD32) ^ hi);
}

/* j-th 64-bit random number: two consecutive 32-bit ones, high word first. */
uint64_t orc_draw64(uint64_t key, uint32_t j)
{
    return ((uint64_t)orc_draw32(key, 2u * j) << 32) | (uint64_t)orc_draw32(key, 2u * j + 1u);
}

/* Map a uniform 32-bit x to [0, m): floor(x * m / 2^32). */
uint32_t orc_bounded32(uint32_t x, uint32_t m)
{
    return (uint32_t)(((uint64_t)x * (uint64_t)m) >> 32);
}

/* Map a uniform 64-bit x to [0, W): floor(x * W / 2^64). */
uint64_t orc_bounded64(uint64_t x, uint64_t W)
{
    return (uint64_t)(((unsigned __int128)x * (unsigned __int128)W) >> 64);
}

/* ------------------------------------------------------------------ */
/* SAMPLE for one GraphSAGE row                                        */
/* ------------------------------------------------------------------ */

/*
 * Sec. 4.1.2: s distinct positions out of deg equally weighted ones (deg > s).
 * Draw j is an integer r in [0, deg - j): the index of the pick among the
 * positions NOT yet chosen, in ascending order (that is what ITS returns on the
 * 0/1 weight vector whose chosen entries were zeroed: the prefix sum at an
 * unchosen position p equals 1 + number of unchosen positions before p).
 * Walking the chosen positions in ascending order and stepping r over each one
 * that is <= r turns that index into the position itself.
 * `chosen` (length s) comes back sorted ascending.
 */
void orc_its_distinct(uint64_t key, uint32_t deg, int32_t s, uint32_t *chosen)
{
    for (int32_t j = 0; j < s; ++j) {
        uint32_t r = orc_bounded32(orc_draw32(key, (uint32_t)j), deg - (uint32_t)j);
        int32_t t = 0;
        while (t < j && r >= chosen[t]) {
            ++r;
            ++t;
        }
        for (int32_t q = j; q > t; --q)
            chosen[q] = chosen[q - 1];
        chosen[t] = r;
    }
}

/*
 * Variant ORC_REPLACE of Sec. 4.1.2: the s draws are independent, each one an
 * integer in [0, deg) (ITS on the unit weights, nothing zeroed, no repetition
 * when two draws coincide).  The nonzeros of the sampled row are the distinct
 * picks: `chosen` receives them sorted ascending, the count is returned
 * (1 <= count <= min(s, deg) for deg >= 1).
 */
int32_t orc_its_replace(uint64_t key, uint32_t deg, int32_t s, uint32_t *chosen)
{
    int32_t c = 0;
    for (int32_t j = 0; j < s; ++j) {
        const uint32_t r = orc_bounded32(orc_draw32(key, (uint32_t)j), deg);
        int32_t t = 0;
        while (t < c && chosen[t] < r)
            ++t;
        if (t < c && chosen[t] == r)
            continue; /* this position already is a nonzero of the row */
        for (int32_t q = c; q > t; --q)
            chosen[q] = chosen[q - 1];
        chosen[t] = r;
        ++c;
    }
    return c;
}

#define ORC_UNION_DST 1 /* columns = sampled vertices and the frontier itself */
#define ORC_REPLACE 2   /* independent draws, distinct picks kept              */

/* ------------------------------------------------------------------ */
/* Result containers                                                   */
/* ------------------------------------------------------------------ */

typedef struct {
    int64_t rows, nnz, ncols, pnnz;
    int64_t *mb_rowoff;  /* k+1 : rows of minibatch i are [mb_rowoff[i], mb_rowoff[i+1]) */
    int32_t *row_vertex; /* rows: global vertex of each stacked row (the frontier)       */
    int64_t *rowptr;     /* rows+1                                                        */
    int32_t *col;        /* nnz : column index local to the row's minibatch              */
    int64_t *mb_coloff;  /* k+1 : columns of minibatch i                                 */
    int32_t *col_vertex; /* ncols: global vertex of each local column, ascending per mb  */
    int64_t *p_off;      /* k+1 : LADIES only, the row of P of each minibatch            */
    int32_t *p_col;      /* pnnz: columns of P ascending                                 */
    uint32_t *p_cnt;     /* pnnz: e_v                                                    */
    int32_t *row_self;   /* rows: ORC_UNION_DST only, local column of the row's own vertex */
} orc_hop;

typedef struct {
    int32_t k, L;
    orc_hop *hop;
} orc_result;

/* one minibatch, one hop, before stacking */
typedef struct {
    int64_t rows, nnz, ncols, pnnz;
    int32_t *row_vertex;
    int64_t *rowptr;
    int32_t *col;
    int32_t *col_vertex;
    int32_t *p_col;
    uint32_t *p_cnt;
    int32_t *row_self;
} mb_hop;

static void mb_hop_free(mb_hop *m)
{
    free(m->row_vertex);
    free(m->rowptr);
    free(m->col);
    free(m->col_vertex);
    free(m->p_col);
    free(m->p_cnt);
    free(m->row_self);
    memset(m, 0, sizeof(*m));
}

static void *xmalloc(size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p)
        abort();
    return p;
}

static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* sorted distinct copy of v[0..m) ; returns the count */
static int64_t sorted_unique(const int32_t *v, int64_t m, int32_t **out)
{
    int32_t *u = (int32_t *)xmalloc((size_t)m * sizeof(int32_t));
    memcpy(u, v, (size_t)m * sizeof(int32_t));
    qsort(u, (size_t)m, sizeof(int32_t), cmp_i32);
    int64_t c = 0;
    for (int64_t i = 0; i < m; ++i)
        if (c == 0 || u[c - 1] != u[i])
            u[c++] = u[i];
    *out = u;
    return c;
}

/* index of x in the sorted distinct array u[0..c), or -1 */
static int64_t find_sorted(const int32_t *u, int64_t c, int32_t x)
{
    int64_t lo = 0, hi = c;
    while (lo < hi) {
        int64_t mid = lo + (hi - lo) / 2;
        if (u[mid] < x)
            lo = mid + 1;
        else
            hi = mid;
    }
    return (lo < c && u[lo] == x) ? lo : -1;
}

/* every id in [0,n) and no id twice: Q^L has one nonzero per batch vertex */
static int batch_is_valid(const int32_t *batch, int32_t b, int64_t n)
{
    int32_t *u;
    for (int32_t i = 0; i < b; ++i)
        if (batch[i] < 0 || (int64_t)batch[i] >= n)
            return 0;
    int64_t c = sorted_unique(batch, b, &u);
    free(u);
    return c == b;
}

/* ------------------------------------------------------------------ */
/* GraphSAGE, one minibatch (Sec. 4.1; Alg. 1 with L iterations)       */
/* ------------------------------------------------------------------ */

static void nodewise_one(const int64_t *A_rowptr, const int32_t *A_col, const int32_t *batch, int32_t b,
                         const int32_t *fanouts, int32_t L, uint64_t seed, uint32_t mb, int variant, mb_hop *out)
{
    int64_t nF = b;
    int32_t *F = (int32_t *)xmalloc((size_t)nF * sizeof(int32_t));
    memcpy(F, batch, (size_t)nF * sizeof(int32_t));

    for (int32_t h = 0; h < L; ++h) {
        const int32_t s = fanouts[h];
        mb_hop *o = &out[h];
        o->rows = nF;
        o->row_vertex = F;

        /* P = Q A: row r of P is the neighbour list of F[r].  SAMPLE: the nonzeros of Q', as global
         * vertex ids, ascending within a row; at most min(deg, s) of them (exactly that many unless
         * the draws are independent) */
        o->rowptr = (int64_t *)xmalloc((size_t)(nF + 1) * sizeof(int64_t));
        o->rowptr[0] = 0;
        int64_t room = nF; /* the frontier itself (ORC_UNION_DST) + at most min(deg, s) per row */
        for (int64_t r = 0; r < nF; ++r) {
            const int64_t deg = A_rowptr[F[r] + 1] - A_rowptr[F[r]];
            room += deg < s ? deg : s;
        }
        int32_t *picked = (int32_t *)xmalloc((size_t)room * sizeof(int32_t));
        uint32_t *chosen = (uint32_t *)xmalloc((size_t)(s > 0 ? s : 1) * sizeof(uint32_t));
        for (int64_t r = 0; r < nF; ++r) {
            const int32_t v = F[r];
            const int64_t beg = A_rowptr[v];
            const int64_t deg = A_rowptr[v + 1] - beg;
            int32_t *dst = picked + o->rowptr[r];
            int64_t len;
            if (variant & ORC_REPLACE) {
                len = deg > 0 ? orc_its_replace(orc_rowkey(seed, h, mb, (uint32_t)v), (uint32_t)deg, s, chosen) : 0;
                for (int64_t t = 0; t < len; ++t)
                    dst[t] = A_col[beg + chosen[t]];
            } else if (deg <= s) {
                len = deg;
                for (int64_t t = 0; t < deg; ++t)
                    dst[t] = A_col[beg + t];
            } else {
                len = s;
                orc_its_distinct(orc_rowkey(seed, h, mb, (uint32_t)v), (uint32_t)deg, s, chosen);
                for (int32_t t = 0; t < s; ++t)
                    dst[t] = A_col[beg + chosen[t]];
            }
            o->rowptr[r + 1] = o->rowptr[r] + len;
        }
        o->nnz = o->rowptr[nF];
        free(chosen);

        /* EXTRACT: drop the empty columns of Q' -> local column = rank among the distinct ids
         * (with ORC_UNION_DST the frontier's own vertices count as nonempty columns too) */
        int64_t ncand = o->nnz;
        if (variant & ORC_UNION_DST) {
            memcpy(picked + ncand, F, (size_t)nF * sizeof(int32_t));
            ncand += nF;
        }
        o->ncols = sorted_unique(picked, ncand, &o->col_vertex);
        o->col = (int32_t *)xmalloc((size_t)o->nnz * sizeof(int32_t));
        for (int64_t e = 0; e < o->nnz; ++e)
            o->col[e] = (int32_t)find_sorted(o->col_vertex, o->ncols, picked[e]);
        if (variant & ORC_UNION_DST) {
            o->row_self = (int32_t *)xmalloc((size_t)nF * sizeof(int32_t));
            for (int64_t r = 0; r < nF; ++r)
                o->row_self[r] = (int32_t)find_sorted(o->col_vertex, o->ncols, F[r]);
        }
        free(picked);

        /* next Q: one row per distinct sampled vertex */
        nF = o->ncols;
        F = (int32_t *)xmalloc((size_t)nF * sizeof(int32_t));
        memcpy(F, o->col_vertex, (size_t)nF * sizeof(int32_t));
    }
    free(F);
}

/* ------------------------------------------------------------------ */
/* LADIES, one minibatch (Sec. 4.2)                                    */
/* ------------------------------------------------------------------ */

static void ladies_one(const int64_t *A_rowptr, const int32_t *A_col, const int32_t *batch, int32_t b,
                       const int32_t *s_per_layer, int32_t L, uint64_t seed, uint32_t mb, int squared, mb_hop *out)
{
    int64_t nF = b;
    int32_t *F = (int32_t *)xmalloc((size_t)nF * sizeof(int32_t));
    memcpy(F, batch, (size_t)nF * sizeof(int32_t));

    for (int32_t h = 0; h < L; ++h) {
        const int32_t s = s_per_layer[h];
        mb_hop *o = &out[h];
        o->rows = nF;
        o->row_vertex = F;

        /* P = Q A with Q the indicator row of F: multiset union of the neighbour lists,
         * then e_v = multiplicity of v */
        int64_t D = 0;
        for (int64_t r = 0; r < nF; ++r)
            D += A_rowptr[F[r] + 1] - A_rowptr[F[r]];
        int32_t *gathered = (int32_t *)xmalloc((size_t)D * sizeof(int32_t));
        int64_t g = 0;
        for (int64_t r = 0; r < nF; ++r)
            for (int64_t e = A_rowptr[F[r]]; e < A_rowptr[F[r] + 1]; ++e)
                gathered[g++] = A_col[e];
        qsort(gathered, (size_t)D, sizeof(int32_t), cmp_i32);
        int64_t C = 0;
        for (int64_t i = 0; i < D; ++i)
            if (i == 0 || gathered[i] != gathered[i - 1])
                ++C;
        o->pnnz = C;
        o->p_col = (int32_t *)xmalloc((size_t)C * sizeof(int32_t));
        o->p_cnt = (uint32_t *)xmalloc((size_t)C * sizeof(uint32_t));
        C = 0;
        for (int64_t i = 0; i < D; ++i) {
            if (i == 0 || gathered[i] != gathered[i - 1]) {
                o->p_col[C] = gathered[i];
                o->p_cnt[C] = 1;
                ++C;
            } else {
                ++o->p_cnt[C - 1];
            }
        }
        free(gathered);

        /* NORM kept implicit: integer weights, inclusive prefix sum, W = row sum */
        uint64_t *prefix = (uint64_t *)xmalloc((size_t)C * sizeof(uint64_t));
        uint64_t W = 0;
        for (int64_t t = 0; t < C; ++t) {
            uint64_t w = o->p_cnt[t];
            W += squared ? w * w : w;
            prefix[t] = W;
        }

        /* SAMPLE: s draws with replacement; pick = smallest t with prefix[t] > r */
        int64_t npick = (W > 0) ? s : 0;
        int32_t *picks = (int32_t *)xmalloc((size_t)npick * sizeof(int32_t));
        const uint64_t key = orc_rowkey(seed, h, mb, ORC_NOVERTEX);
        for (int64_t j = 0; j < npick; ++j) {
            uint64_t r = orc_bounded64(orc_draw64(key, (uint32_t)j), W);
            int64_t lo = 0, hi = C - 1;
            while (lo < hi) {
                int64_t mid = lo + (hi - lo) / 2;
                if (prefix[mid] > r)
                    hi = mid;
                else
                    lo = mid + 1;
            }
            picks[j] = o->p_col[lo];
        }
        free(prefix);
        o->ncols = sorted_unique(picks, npick, &o->col_vertex);
        free(picks);

        /* EXTRACT: rows of A for F (Q_R A), then only the sampled columns (.. Q_C),
         * columns relabelled to their index in the sampled set */
        o->rowptr = (int64_t *)xmalloc((size_t)(nF + 1) * sizeof(int64_t));
        o->rowptr[0] = 0;
        for (int64_t r = 0; r < nF; ++r) {
            int64_t c = 0;
            for (int64_t e = A_rowptr[F[r]]; e < A_rowptr[F[r] + 1]; ++e)
                if (find_sorted(o->col_vertex, o->ncols, A_col[e]) >= 0)
                    ++c;
            o->rowptr[r + 1] = o->rowptr[r] + c;
        }
        o->nnz = o->rowptr[nF];
        o->col = (int32_t *)xmalloc((size_t)o->nnz * sizeof(int32_t));
        int64_t w = 0;
        for (int64_t r = 0; r < nF; ++r)
            for (int64_t e = A_rowptr[F[r]]; e < A_rowptr[F[r] + 1]; ++e) {
                int64_t c = find_sorted(o->col_vertex, o->ncols, A_col[e]);
                if (c >= 0)
                    o->col[w++] = (int32_t)c;
            }

        nF = o->ncols;
        F = (int32_t *)xmalloc((size_t)nF * sizeof(int32_t));
        memcpy(F, o->col_vertex, (size_t)nF * sizeof(int32_t));
    }
    free(F);
}

/* ------------------------------------------------------------------ */
/* Bulk: stack the k minibatches (Eq. 1)                               */
/* ------------------------------------------------------------------ */

static orc_result *stack_minibatches(mb_hop *per, int32_t k, int32_t L, int with_p, int with_self)
{
    orc_result *res = (orc_result *)xmalloc(sizeof(orc_result));
    res->k = k;
    res->L = L;
    res->hop = (orc_hop *)xmalloc((size_t)L * sizeof(orc_hop));
    memset(res->hop, 0, (size_t)L * sizeof(orc_hop));
    for (int32_t h = 0; h < L; ++h) {
        orc_hop *o = &res->hop[h];
        o->mb_rowoff = (int64_t *)xmalloc((size_t)(k + 1) * sizeof(int64_t));
        o->mb_coloff = (int64_t *)xmalloc((size_t)(k + 1) * sizeof(int64_t));
        o->p_off = (int64_t *)xmalloc((size_t)(k + 1) * sizeof(int64_t));
        o->mb_rowoff[0] = o->mb_coloff[0] = o->p_off[0] = 0;
        int64_t nnz = 0;
        for (int32_t i = 0; i < k; ++i) {
            const mb_hop *m = &per[(size_t)i * L + h];
            o->mb_rowoff[i + 1] = o->mb_rowoff[i] + m->rows;
            o->mb_coloff[i + 1] = o->mb_coloff[i] + m->ncols;
            o->p_off[i + 1] = o->p_off[i] + m->pnnz;
            nnz += m->nnz;
        }
        o->rows = o->mb_rowoff[k];
        o->ncols = o->mb_coloff[k];
        o->pnnz = o->p_off[k];
        o->nnz = nnz;
        o->row_vertex = (int32_t *)xmalloc((size_t)o->rows * sizeof(int32_t));
        o->rowptr = (int64_t *)xmalloc((size_t)(o->rows + 1) * sizeof(int64_t));
        o->col = (int32_t *)xmalloc((size_t)o->nnz * sizeof(int32_t));
        o->col_vertex = (int32_t *)xmalloc((size_t)o->ncols * sizeof(int32_t));
        if (with_p) {
            o->p_col = (int32_t *)xmalloc((size_t)o->pnnz * sizeof(int32_t));
            o->p_cnt = (uint32_t *)xmalloc((size_t)o->pnnz * sizeof(uint32_t));
        }
        if (with_self)
            o->row_self = (int32_t *)xmalloc((size_t)o->rows * sizeof(int32_t));
        int64_t e0 = 0;
        o->rowptr[0] = 0;
        for (int32_t i = 0; i < k; ++i) {
            const mb_hop *m = &per[(size_t)i * L + h];
            const int64_t r0 = o->mb_rowoff[i];
            memcpy(o->row_vertex + r0, m->row_vertex, (size_t)m->rows * sizeof(int32_t));
            if (with_self)
                memcpy(o->row_self + r0, m->row_self, (size_t)m->rows * sizeof(int32_t));
            for (int64_t r = 0; r < m->rows; ++r)
                o->rowptr[r0 + r + 1] = e0 + m->rowptr[r + 1];
            memcpy(o->col + e0, m->col, (size_t)m->nnz * sizeof(int32_t));
            e0 += m->nnz;
            memcpy(o->col_vertex + o->mb_coloff[i], m->col_vertex, (size_t)m->ncols * sizeof(int32_t));
            if (with_p) {
                memcpy(o->p_col + o->p_off[i], m->p_col, (size_t)m->pnnz * sizeof(int32_t));
                memcpy(o->p_cnt + o->p_off[i], m->p_cnt, (size_t)m->pnnz * sizeof(uint32_t));
            }
        }
    }
    return res;
}

static int check_args(const int64_t *rowptr, const int32_t *col, int64_t n, const int32_t *batches, int32_t k, int32_t b,
                      const int32_t *param, int32_t L)
{
    if (!rowptr || (!col && rowptr[n] > 0) || !batches || !param || n < 0 || k < 1 || b < 1 || L < 1)
        return -1;
    for (int32_t h = 0; h < L; ++h)
        if (param[h] < 1)
            return -1;
    for (int32_t i = 0; i < k; ++i)
        if (!batch_is_valid(batches + (size_t)i * b, b, n))
            return -2;
    return 0;
}

/*
 * Bulk GraphSAGE sampling of k minibatches of b seed vertices each.
 * batches: k*b vertex ids, row-major.  fanouts[h] is s at hop h (hop 0 = the seeds,
 * i.e. the paper's layer L).  Minibatch i uses random-stream index mb_base + i.
 * Returns 0, -1 (bad argument) or -2 (seed out of range / repeated in a minibatch).
 */
int orc_sample_nodewise_variant(const int64_t *rowptr, const int32_t *col, int64_t n, const int32_t *batches,
                                int32_t k, int32_t b, const int32_t *fanouts, int32_t L, uint64_t seed,
                                int32_t mb_base, int variant, orc_result **out)
{
    int rc = check_args(rowptr, col, n, batches, k, b, fanouts, L);
    if (rc)
        return rc;
    if (variant & ~(ORC_UNION_DST | ORC_REPLACE))
        return -1;
    mb_hop *per = (mb_hop *)xmalloc((size_t)k * L * sizeof(mb_hop));
    memset(per, 0, (size_t)k * L * sizeof(mb_hop));
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < k; ++i)
        nodewise_one(rowptr, col, batches + (size_t)i * b, b, fanouts, L, seed, (uint32_t)(mb_base + i), variant,
                     per + (size_t)i * L);
    *out = stack_minibatches(per, k, L, 0, variant & ORC_UNION_DST);
    for (size_t q = 0; q < (size_t)k * L; ++q)
        mb_hop_free(&per[q]);
    free(per);
    return 0;
}

/* the method as the paper states it: no variant */
int orc_sample_nodewise(const int64_t *rowptr, const int32_t *col, int64_t n, const int32_t *batches, int32_t k,
                        int32_t b, const int32_t *fanouts, int32_t L, uint64_t seed, int32_t mb_base, orc_result **out)
{
    return orc_sample_nodewise_variant(rowptr, col, n, batches, k, b, fanouts, L, seed, mb_base, 0, out);
}

/*
 * Bulk LADIES sampling.  s_per_layer[h] draws at hop h; squared != 0 weights
 * column v by e_v^2 instead of e_v.
 */
int orc_sample_ladies(const int64_t *rowptr, const int32_t *col, int64_t n, const int32_t *batches, int32_t k,
                      int32_t b, const int32_t *s_per_layer, int32_t L, uint64_t seed, int32_t mb_base, int squared,
                      orc_result **out)
{
    int rc = check_args(rowptr, col, n, batches, k, b, s_per_layer, L);
    if (rc)
        return rc;
    mb_hop *per = (mb_hop *)xmalloc((size_t)k * L * sizeof(mb_hop));
    memset(per, 0, (size_t)k * L * sizeof(mb_hop));
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t i = 0; i < k; ++i)
        ladies_one(rowptr, col, batches + (size_t)i * b, b, s_per_layer, L, seed, (uint32_t)(mb_base + i), squared,
                   per + (size_t)i * L);
    *out = stack_minibatches(per, k, L, 1, 0);
    for (size_t q = 0; q < (size_t)k * L; ++q)
        mb_hop_free(&per[q]);
    free(per);
    return 0;
}

const orc_hop *orc_result_hop(const orc_result *res, int32_t hop)
{
    if (!res || hop < 0 || hop >= res->L)
        return NULL;
    return &res->hop[hop];
}

void orc_result_free(orc_result *res)
{
    if (!res)
        return;
    for (int32_t h = 0; h < res->L; ++h) {
        orc_hop *o = &res->hop[h];
        free(o->mb_rowoff);
        free(o->row_vertex);
        free(o->rowptr);
        free(o->col);
        free(o->mb_coloff);
        free(o->col_vertex);
        free(o->p_off);
        free(o->p_col);
        free(o->p_cnt);
        free(o->row_self);
    }
    free(res->hop);
    free(res);
}

/* threads used by the loop over minibatches (1 when built without OpenMP) */
int orc_set_threads(int nthreads)
{
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
    return omp_get_max_threads();
#else
    (void)nthreads;
    return 1;
#endif
}

/*
 * Feature fetching, the part one GPU does (Sec. 6.2): H_i holds the rows of the feature matrix H that
 * belong to the vertices of a minibatch's last frontier, in frontier order.  H is n x f, row-major.
 * Returns 0, or -2 when an id lies outside [0, n) (such rows are written as zeros).
 */
int orc_fetch_features(const float *H, int64_t n, int32_t f, const int32_t *ids, int64_t m, float *out)
{
    int rc = 0;
    for (int64_t j = 0; j < m; ++j) {
        const int64_t v = ids[j];
        for (int32_t x = 0; x < f; ++x) {
            if (v < 0 || v >= n) {
                out[j * f + x] = 0.0f;
                rc = -2;
            } else {
                out[j * f + x] = H[v * f + x];
            }
        }
    }
    return rc;
}

/*
 * Forward neighbourhood aggregation of one hop (Sec. 6.2: an SpMM between a minibatch's sampled adjacency
 * matrix A_i and the feature rows H_i of its columns), written for the stacked result: row r of minibatch i
 * has entries e in [rowptr[r], rowptr[r+1]) whose local columns col[e] index the minibatch's own block of
 * X, which starts at row mb_coloff[i].  out[r, :] = sum over e of X[mb_coloff[i] + col[e], :], divided by
 * the number of entries when mean != 0 (all entries of A_i are 1).  Accumulated in double in entry order and
 * rounded to float once; a row without entries gives zeros.
 */
void orc_aggregate(const int64_t *mb_rowoff, int32_t k, const int64_t *rowptr, const int32_t *col,
                   const int64_t *mb_coloff, const float *X, int32_t f, int mean, float *out)
{
    for (int32_t i = 0; i < k; ++i) {
        for (int64_t r = mb_rowoff[i]; r < mb_rowoff[i + 1]; ++r) {
            const int64_t len = rowptr[r + 1] - rowptr[r];
            for (int32_t x = 0; x < f; ++x) {
                double acc = 0.0;
                for (int64_t e = rowptr[r]; e < rowptr[r + 1]; ++e)
                    acc += (double)X[(mb_coloff[i] + col[e]) * f + x];
                if (mean && len > 0)
                    acc /= (double)len;
                out[r * f + x] = (float)acc;
            }
        }
    }
}
