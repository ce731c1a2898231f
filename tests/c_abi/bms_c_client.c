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
    if (argc != 3 && argc != 4) {
        fprintf(stderr, "usage: %s problem.bin result.bin [flags]\n", argv[0]);
        return 2;
    }
    const uint32_t flags = argc == 4 ? (uint32_t)strtoul(argv[3], NULL, 10) : 0u;
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
