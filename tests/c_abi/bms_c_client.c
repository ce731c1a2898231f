/*
 * A client of libbms.so written in plain C: proves that the boundary needs nothing but include/bms.h, host
 * arrays and the HIP runtime's memory copies.  Reads a problem from a binary file, samples it node-wise
 * through the C ABI and writes every array of every hop to a second file (tests/test_gpu_c_abi.py compares
 * that file with the oracle).
 *
 *   in : int64 n, nnz, k, b, L, seed; int64 rowptr[n+1]; int32 col[nnz]; int32 batches[k*b]; int32 fanouts[L]
 *   out: per hop  int64 rows, nnz, ncols; int64 mb_rowoff[k+1]; int32 row_vertex[rows]; int64 rowptr[rows+1];
 *                 int32 col[nnz]; int64 mb_coloff[k+1]; int32 col_vertex[ncols]; with BMS_UNION_DST int32 row_self[rows]
 * An optional third argument gives bms_opts.flags (decimal), e.g. 128 for BMS_UNION_DST.
 * With a fourth argument ("consumers") the file continues with what the other entry points give on the same problem:
 *   per hop, per minibatch (bms_result_minibatch): int64 rows, nnz, ncols, row0, edge0, col0
 *   bms_fetch_features of the last hop's columns from H[v, x] = (31 v + 7 x) mod 997, f = 8: float X[ncols * f]
 *   bms_aggregate_hop of the last hop over X (sums): float out[rows * f]
 *   bms_sample_ladies with s = 8 * fanouts[h]: per hop as above, then int64 pnnz; int64 p_off[k+1]; int32 p_col[pnnz];
 *                 uint32 p_cnt[pnnz]
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "bms.h"

static void *read_array(FILE *f, size_t count, size_t size)
{
    void *p = malloc(count * size + 1);
    if (!p || fread(p, size, count, f) != count) {
        fprintf(stderr, "short read\n");
        exit(2);
    }
    return p;
}

static void dump(FILE *f, const void *dev, size_t count, size_t size)
{
    void *host = malloc(count * size + 1);
    if (!host || (count && hipMemcpy(host, dev, count * size, hipMemcpyDeviceToHost) != hipSuccess)) {
        fprintf(stderr, "copy back failed\n");
        exit(3);
    }
    fwrite(host, size, count, f);
    free(host);
}

int main(int argc, char **argv)
{
    if (argc < 3 || argc > 5) {
        fprintf(stderr, "usage: %s problem.bin result.bin [flags [consumers]]\n", argv[0]);
        return 2;
    }
    const uint32_t flags = argc >= 4 ? (uint32_t)strtoul(argv[3], NULL, 10) : 0u;
    const int consumers = argc == 5;
    FILE *in = fopen(argv[1], "rb");
    if (!in)
        return 2;
    int64_t head[6];
    if (fread(head, sizeof(int64_t), 6, in) != 6)
        return 2;
    const int64_t n = head[0], nnz = head[1];
    const int32_t k = (int32_t)head[2], b = (int32_t)head[3], L = (int32_t)head[4];
    const uint64_t seed = (uint64_t)head[5];
    int64_t *rowptr = read_array(in, (size_t)n + 1, sizeof(int64_t));
    int32_t *col = read_array(in, (size_t)nnz, sizeof(int32_t));
    int32_t *batches = read_array(in, (size_t)k * b, sizeof(int32_t));
    int32_t *fanouts = read_array(in, (size_t)L, sizeof(int32_t));
    fclose(in);

    bms_csr *csr = NULL;
    int rc = bms_csr_load(rowptr, col, n, nnz, BMS_HOST, &csr);
    if (rc != BMS_OK) {
        fprintf(stderr, "bms_csr_load: %s (%s)\n", bms_strerror(rc), bms_last_error());
        return 1;
    }
    bms_opts opts = {0};
    opts.flags = flags;
    bms_result *res = NULL;
    rc = bms_sample_nodewise(csr, batches, k, b, fanouts, L, seed, &opts, &res);
    if (rc != BMS_OK) {
        fprintf(stderr, "bms_sample_nodewise: %s (%s)\n", bms_strerror(rc), bms_last_error());
        return 1;
    }
    /* a second call into the same result: the steady state a training loop runs in */
    opts.recycle = res;
    rc = bms_sample_nodewise(csr, batches, k, b, fanouts, L, seed, &opts, &res);
    if (rc != BMS_OK) {
        fprintf(stderr, "recycled call: %s (%s)\n", bms_strerror(rc), bms_last_error());
        return 1;
    }
    FILE *out = fopen(argv[2], "wb");
    if (!out)
        return 2;
    for (int32_t h = 0; h < L; ++h) {
        bms_hop_view v;
        if (bms_result_hop(res, h, &v) != BMS_OK)
            return 1;
        const int64_t sizes[3] = {v.rows, v.nnz, v.ncols};
        fwrite(sizes, sizeof(int64_t), 3, out);
        dump(out, v.mb_rowoff, (size_t)k + 1, sizeof(int64_t));
        dump(out, v.row_vertex, (size_t)v.rows, sizeof(int32_t));
        dump(out, v.rowptr, (size_t)v.rows + 1, sizeof(int64_t));
        dump(out, v.col, (size_t)v.nnz, sizeof(int32_t));
        dump(out, v.mb_coloff, (size_t)k + 1, sizeof(int64_t));
        dump(out, v.col_vertex, (size_t)v.ncols, sizeof(int32_t));
        if ((flags & BMS_UNION_DST) != 0) {
            if (!v.row_self)
                return 1;
            dump(out, v.row_self, (size_t)v.rows, sizeof(int32_t));
        } else if (v.row_self) {
            return 1;
        }
    }
    if (consumers) {
        enum { F = 8 };
        for (int32_t h = 0; h < L; ++h)
            for (int32_t i = 0; i < k; ++i) {
                bms_mb_view m;
                if (bms_result_minibatch(res, h, i, &m) != BMS_OK)
                    return 1;
                const int64_t six[6] = {m.rows, m.nnz, m.ncols, m.row0, m.edge0, m.col0};
                fwrite(six, sizeof(int64_t), 6, out);
            }
        bms_hop_view last;
        if (bms_result_hop(res, L - 1, &last) != BMS_OK)
            return 1;
        float *H_host = malloc((size_t)n * F * sizeof(float) + 1), *H = NULL, *X = NULL, *agg = NULL;
        for (int64_t v = 0; v < n; ++v)
            for (int x = 0; x < F; ++x)
                H_host[v * F + x] = (float)((31 * v + 7 * x) % 997);
        if (hipMalloc((void **)&H, (size_t)n * F * sizeof(float) + 4) != hipSuccess ||
            hipMalloc((void **)&X, (size_t)last.ncols * F * sizeof(float) + 4) != hipSuccess ||
            hipMalloc((void **)&agg, (size_t)last.rows * F * sizeof(float) + 4) != hipSuccess ||
            hipMemcpy(H, H_host, (size_t)n * F * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
            return 3;
        rc = bms_fetch_features(H, n, F, last.col_vertex, last.ncols, X, NULL);
        if (rc != BMS_OK) {
            fprintf(stderr, "bms_fetch_features: %s (%s)\n", bms_strerror(rc), bms_last_error());
            return 1;
        }
        dump(out, X, (size_t)last.ncols * F, sizeof(float));
        rc = bms_aggregate_hop(res, L - 1, X, F, 0, agg, NULL);
        if (rc != BMS_OK || hipDeviceSynchronize() != hipSuccess) {
            fprintf(stderr, "bms_aggregate_hop: %s (%s)\n", bms_strerror(rc), bms_last_error());
            return 1;
        }
        dump(out, agg, (size_t)last.rows * F, sizeof(float));
        (void)hipFree(H);
        (void)hipFree(X);
        (void)hipFree(agg);
        free(H_host);
        int32_t *s_per_layer = malloc((size_t)L * sizeof(int32_t));
        for (int32_t h = 0; h < L; ++h)
            s_per_layer[h] = 8 * fanouts[h];
        bms_opts lopts = {0};
        bms_result *lad = NULL;
        rc = bms_sample_ladies(csr, batches, k, b, s_per_layer, L, seed, &lopts, &lad);
        if (rc != BMS_OK) {
            fprintf(stderr, "bms_sample_ladies: %s (%s)\n", bms_strerror(rc), bms_last_error());
            return 1;
        }
        for (int32_t h = 0; h < L; ++h) {
            bms_hop_view v;
            if (bms_result_hop(lad, h, &v) != BMS_OK || !v.p_off)
                return 1;
            const int64_t sizes[3] = {v.rows, v.nnz, v.ncols};
            fwrite(sizes, sizeof(int64_t), 3, out);
            dump(out, v.mb_rowoff, (size_t)k + 1, sizeof(int64_t));
            dump(out, v.row_vertex, (size_t)v.rows, sizeof(int32_t));
            dump(out, v.rowptr, (size_t)v.rows + 1, sizeof(int64_t));
            dump(out, v.col, (size_t)v.nnz, sizeof(int32_t));
            dump(out, v.mb_coloff, (size_t)k + 1, sizeof(int64_t));
            dump(out, v.col_vertex, (size_t)v.ncols, sizeof(int32_t));
            fwrite(&v.pnnz, sizeof(int64_t), 1, out);
            dump(out, v.p_off, (size_t)k + 1, sizeof(int64_t));
            dump(out, v.p_col, (size_t)v.pnnz, sizeof(int32_t));
            dump(out, v.p_cnt, (size_t)v.pnnz, sizeof(uint32_t));
        }
        bms_free(lad);
        free(s_per_layer);
    }
    fclose(out);
    /* an invalid batch must come back as an error code, not as a crash */
    batches[1] = batches[0];
    opts.recycle = NULL;
    bms_result *bad = NULL;
    rc = bms_sample_nodewise(csr, batches, k, b, fanouts, L, seed, &opts, &bad);
    if (b > 1 && (rc != BMS_ERANGE || bad != NULL)) {
        fprintf(stderr, "repeated seed gave %d\n", rc);
        return 1;
    }
    bms_free(res);
    bms_free(csr);
    free(rowptr);
    free(col);
    free(batches);
    free(fanouts);
    printf("ok\n");
    return 0;
}
