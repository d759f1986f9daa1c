/*
 * CPU oracle for the unaligned block-pruned (UBP) sparse x dense product.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or import
 * this file; only the tests, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What it computes is the plain definition the paper's inference kernel reaches by a
 * faster route (Section 3.3 and Section 4.2: the WROS dataflow only reorders weights
 * and loop iterations, it changes no value):
 *
 *   1. validate the block list: every block inside the matrix (the edge rule of Eq. 1)
 *      and no two blocks sharing a cell (the non-overlap constraint of Eq. 2);
 *   2. densify: Wd = 0; for every block, copy its bh x bw cells from W (every cell that
 *      lies in no kept block is zero, Section 3.1);
 *   3. Y[i][j] = sum_k Wd[i][k] * X[k][j], a naive loop nest in double precision that
 *      skips nothing (the worked sum for O_23 in Section 3.3 is one instance of it).
 *
 * It also writes out the sparse format of Section 4.2 (block values rotated so that the
 * weight of matrix row i sits in slot i mod bh; `indices`; `indptr`) straight from its
 * definition, for bit-exact comparison with the library's packer.  Readings taken where
 * the paper's format picture is unavailable: `indptr` has one entry per start row
 * (Section 3.3: the tile row index advances by 1) plus the end sentinel, i.e.
 * M - bh + 2 entries; blocks with equal start row are ordered by ascending column
 * origin; a block of width bw > 1 stores its bw columns one after the other, each as bh
 * rotated slots.
 *
 * All floating-point inputs arrive as double (the caller converts the already-rounded
 * fp32 / fp16 / bf16 values exactly).  Single-threaded on purpose.
 *
 * Pins (tests/test_oracle_pins.py): the paper's N=3 worked example, brute force over
 * blocks on tiny inputs, dense GEMM for an all-blocks-kept W, SciPy BSR for aligned
 * origins, the single-block closed form, X = identity.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_OK = 0, ORC_BAD_ARG = 1, ORC_OUT_OF_BOUNDS = 2, ORC_OVERLAP = 3, ORC_NOMEM = 4 };

/* Paint every block on an M x K byte map; report the first violation.
 * *painted receives the number of kept cells (nb * bh * bw when valid). */
int ubp_oracle_validate(int32_t M, int32_t K, int32_t bh, int32_t bw,
                        const int32_t *blocks, int64_t nb, int64_t *painted)
{
    if (M < 1 || K < 1 || bh < 1 || bw < 1 || nb < 0 || (nb > 0 && !blocks)) return ORC_BAD_ARG;
    unsigned char *map = (unsigned char *)calloc((size_t)M * (size_t)K, 1);
    if (!map) return ORC_NOMEM;
    int64_t cells = 0;
    int rc = ORC_OK;
    for (int64_t b = 0; b < nb && rc == ORC_OK; ++b) {
        int32_t r = blocks[2 * b], c = blocks[2 * b + 1];
        if (r < 0 || c < 0 || (int64_t)r + bh > M || (int64_t)c + bw > K) { rc = ORC_OUT_OF_BOUNDS; break; }
        for (int32_t di = 0; di < bh && rc == ORC_OK; ++di)
            for (int32_t dj = 0; dj < bw; ++dj) {
                unsigned char *cell = &map[(size_t)(r + di) * K + (c + dj)];
                if (*cell) { rc = ORC_OVERLAP; break; }
                *cell = 1;
                ++cells;
            }
    }
    free(map);
    if (painted) *painted = cells;
    return rc;
}

/* Wd (M x K, contiguous) = W restricted to the cells of the blocks, zero elsewhere. */
int ubp_oracle_densify(const double *W, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw,
                       const int32_t *blocks, int64_t nb, double *Wd)
{
    int rc = ubp_oracle_validate(M, K, bh, bw, blocks, nb, NULL);
    if (rc != ORC_OK) return rc;
    for (size_t t = 0; t < (size_t)M * (size_t)K; ++t) Wd[t] = 0.0;
    for (int64_t b = 0; b < nb; ++b) {
        int32_t r = blocks[2 * b], c = blocks[2 * b + 1];
        for (int32_t di = 0; di < bh; ++di)
            for (int32_t dj = 0; dj < bw; ++dj)
                Wd[(size_t)(r + di) * K + (c + dj)] = W[(size_t)(r + di) * ldw + (c + dj)];
    }
    return ORC_OK;
}

/* Y[t][j] = sum_k Wd[rows[t]][k] * X[k][j] for the listed output rows (rows == NULL:
 * all M rows in order).  Yabs, if given, receives sum_k |Wd||X| (the scale against
 * which a componentwise error bound is stated).  No zero is skipped. */
int ubp_oracle_gemm_rows(const double *Wd, const double *X, int64_t ldx, int32_t M, int32_t K, int32_t N,
                         const int32_t *rows, int32_t nrows, double *Y, double *Yabs)
{
    if (!rows) nrows = M;
    for (int32_t t = 0; t < nrows; ++t) {
        int32_t i = rows ? rows[t] : t;
        if (i < 0 || i >= M) return ORC_OUT_OF_BOUNDS;
        double *y = Y + (size_t)t * N;
        double *ya = Yabs ? Yabs + (size_t)t * N : NULL;
        for (int32_t j = 0; j < N; ++j) y[j] = 0.0;
        if (ya) for (int32_t j = 0; j < N; ++j) ya[j] = 0.0;
        for (int32_t k = 0; k < K; ++k) {
            double w = Wd[(size_t)i * K + k];
            double wa = w < 0 ? -w : w;
            const double *x = X + (size_t)k * ldx;
            for (int32_t j = 0; j < N; ++j) y[j] += w * x[j];
            if (ya) for (int32_t j = 0; j < N; ++j) ya[j] += wa * (x[j] < 0 ? -x[j] : x[j]);
        }
    }
    return ORC_OK;
}

/* validate + densify + product, in one call. */
int ubp_oracle_spmm(const double *W, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw,
                    const int32_t *blocks, int64_t nb, const double *X, int64_t ldx, int32_t N,
                    const int32_t *rows, int32_t nrows, double *Y, double *Yabs)
{
    double *Wd = (double *)malloc((size_t)M * (size_t)K * sizeof(double));
    if (!Wd) return ORC_NOMEM;
    int rc = ubp_oracle_densify(W, ldw, M, K, bh, bw, blocks, nb, Wd);
    if (rc == ORC_OK) rc = ubp_oracle_gemm_rows(Wd, X, ldx, M, K, N, rows, nrows, Y, Yabs);
    free(Wd);
    return rc;
}

static int cmp_block(const void *a, const void *b)
{
    const int32_t *p = (const int32_t *)a, *q = (const int32_t *)b;
    if (p[0] != q[0]) return p[0] < q[0] ? -1 : 1;
    if (p[1] != q[1]) return p[1] < q[1] ? -1 : 1;
    return 0;
}

/* The sparse format of Section 4.2, element type opaque (esz bytes, bits copied):
 *   indptr[i], i = 0..M-bh+1 : number of blocks whose start row is < i
 *   indices[b]               : column origin of block b (blocks ordered by start row, then column)
 *   values[((b*bw + q)*bh + s)] = W[rho][c_b + q], rho the row of block b with rho mod bh == s */
int ubp_oracle_pack(const void *W, int64_t esz, int64_t ldw, int32_t M, int32_t K, int32_t bh, int32_t bw,
                    const int32_t *blocks, int64_t nb, int32_t *indptr, int32_t *indices, void *values)
{
    int rc = ubp_oracle_validate(M, K, bh, bw, blocks, nb, NULL);
    if (rc != ORC_OK) return rc;
    int32_t *sorted = (int32_t *)malloc((size_t)(nb > 0 ? nb : 1) * 2 * sizeof(int32_t));
    if (!sorted) return ORC_NOMEM;
    if (nb > 0) memcpy(sorted, blocks, (size_t)nb * 2 * sizeof(int32_t));
    qsort(sorted, (size_t)nb, 2 * sizeof(int32_t), cmp_block);
    int32_t nstart = M - bh + 1;                   /* valid start rows 0 .. M-bh */
    for (int32_t i = 0; i <= nstart; ++i) {
        int64_t cnt = 0;
        for (int64_t b = 0; b < nb; ++b) if (sorted[2 * b] < i) ++cnt;
        indptr[i] = (int32_t)cnt;
    }
    const unsigned char *w = (const unsigned char *)W;
    unsigned char *v = (unsigned char *)values;
    for (int64_t b = 0; b < nb; ++b) {
        int32_t r = sorted[2 * b], c = sorted[2 * b + 1];
        indices[b] = c;
        for (int32_t q = 0; q < bw; ++q)
            for (int32_t di = 0; di < bh; ++di) {
                int32_t rho = r + di, s = rho % bh;
                memcpy(v + (size_t)((b * bw + q) * bh + s) * esz,
                       w + ((size_t)rho * ldw + (c + q)) * esz, (size_t)esz);
            }
    }
    free(sorted);
    return ORC_OK;
}
