/*
 * CPU ORACLE for the MaxK-GNN aggregation path.  TEST INFRASTRUCTURE ONLY:
 * used by tests/, by the smoke check and by the cpu_baseline leg of the
 * benchmark.  The product (the HIP library) never calls, links or imports it,
 * and the two share no code.
 *
 * Every function is the plain definition from the paper, written out with
 * double-precision accumulation, no blocking, no fusion, no reordering:
 *
 *   oracle_topk_cbsr   MaxK nonlinearity + CBSR packing      (Sec. 3.1 definition, Eq. 1; Sec. 3.2 "Forward Computation")
 *   oracle_spgemm_fwd  X_l[i,:] = sum_j A[i,j] * h(X)[j,:]   (Eq. 2 left; Sec. 3.2 row-wise product)
 *   oracle_sspmm_bwd   dXs = (A^T * dX_l) at sp_index        (Eq. 2 right, Eq. 3; Alg. 2 with destination row j)
 *   oracle_spmm        Y = A * H, dense features             (the SpMM the paper compares against, Sec. 5.2)
 *   oracle_cbsr_scatter dH from dXs: MaxK's backward          (Sec. 3.1 definition, part (ii))
 *
 * Readings of points the paper leaves open (each restated where it is used):
 *   - top-k is by signed value, exactly k survive, ties at the k-th value go
 *     to the LOWER column; entries of a CBSR row are stored by ascending column.
 *   - Alg. 2's update is read as dXs[j,t] += e_ij * dX_l[i, sp_index[j,t]]
 *     (destination and index row are the neighbour j, as the prose and the
 *     Fig. 6 walk-through say).
 *   - outputs are overwritten, not accumulated into.
 *
 * Each aggregation also returns the sum of absolute values of the terms of
 * every output element, which the parity bound |err| <= 1e-5*abs + 1e-6 needs.
 *
 * Pins (tests/test_oracle_*.py): dense brute force on tiny graphs, k = dim
 * reduces to SpMM (scipy), identity adjacency, the adjoint identity on a
 * non-symmetric matrix, NumPy stable argsort, hand-worked goldens.
 * Nothing here is "parity unpinned".
 *
 * Plain C + OpenMP over independent outputs.
 * Build: gcc -O2 -fopenmp -shared -fPIC maxk_oracle.c -o liboracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ top-k */

typedef struct {
    float v;
    int32_t c;
} entry_t;

/* order: larger value first (IEEE compare, so -0.0 == +0.0), then lower column */
static int cmp_value_desc_col_asc(const void *pa, const void *pb)
{
    const entry_t *a = (const entry_t *)pa, *b = (const entry_t *)pb;
    if (a->v > b->v) return -1;
    if (a->v < b->v) return 1;
    return (a->c > b->c) - (a->c < b->c);
}

static int cmp_col_asc(const void *pa, const void *pb)
{
    const entry_t *a = (const entry_t *)pa, *b = (const entry_t *)pb;
    return (a->c > b->c) - (a->c < b->c);
}

/*
 * MaxK (Sec. 3.1): keep the k largest entries of every row of H[N x dim];
 * CBSR (Sec. 3.2): sp_index[i,0..k) = kept columns, ascending;
 * sp_data[i,t] = H[i, sp_index[i,t]] (same bits).
 * Returns 0, or -1 if a NaN is met (outside the contract) or arguments are bad.
 */
int oracle_topk_cbsr(const float *H, int64_t N, int32_t dim, int32_t k, float *sp_data, int32_t *sp_index)
{
    if (N < 0 || dim < 1 || k < 1 || k > dim) return -1;
    int bad = 0;
#pragma omp parallel
    {
        entry_t *e = (entry_t *)malloc(sizeof(entry_t) * (size_t)dim);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            const float *row = H + i * (int64_t)dim;
            for (int32_t c = 0; c < dim; ++c) {
                if (row[c] != row[c]) bad = 1;
                e[c].v = row[c];
                e[c].c = c;
            }
            qsort(e, (size_t)dim, sizeof(entry_t), cmp_value_desc_col_asc); /* total order: no ties left */
            qsort(e, (size_t)k, sizeof(entry_t), cmp_col_asc);             /* the k survivors, by column */
            for (int32_t t = 0; t < k; ++t) {
                sp_index[i * (int64_t)k + t] = e[t].c;
                sp_data[i * (int64_t)k + t] = row[e[t].c];
            }
        }
        free(e);
    }
    return bad ? -1 : 0;
}

/* ---------------------------------------------------------------- forward */

/*
 * Row-wise product (Sec. 3.2):  Y[i,c] = sum_{p in row i} val[p] * X[col[p], c],
 * X = the N x dim matrix whose row j holds sp_data[j,t] at column sp_index[j,t]
 * and zero elsewhere.  Yabs[i,c] = the same sum over |terms|.
 * rows == NULL: all rows, outputs are N x dim.  Otherwise outputs are
 * nrows x dim and output row r is graph row rows[r].
 */
int oracle_spgemm_fwd(int64_t N, const int32_t *rowptr, const int32_t *col, const float *val, const float *sp_data,
                      const int32_t *sp_index, int32_t dim, int32_t k, const int64_t *rows, int64_t nrows, double *Y,
                      double *Yabs)
{
    if (N < 0 || dim < 1 || k < 1 || k > dim) return -1;
    if (!rows) nrows = N;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        double *y = Y + r * (int64_t)dim, *ya = Yabs + r * (int64_t)dim;
        for (int32_t c = 0; c < dim; ++c) y[c] = ya[c] = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t j = col[p];
            double a = (double)val[p];
            for (int32_t t = 0; t < k; ++t) {
                double term = a * (double)sp_data[j * k + t];
                int32_t c = sp_index[j * k + t];
                y[c] += term;
                ya[c] += fabs(term);
            }
        }
    }
    return 0;
}

/* Dense-feature SpMM: Y[i,c] = sum_p val[p] * H[col[p], c]  (rows as above) */
int oracle_spmm(int64_t N, const int32_t *rowptr, const int32_t *col, const float *val, const float *H, int32_t dim,
                const int64_t *rows, int64_t nrows, double *Y, double *Yabs)
{
    if (N < 0 || dim < 1) return -1;
    if (!rows) nrows = N;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t r = 0; r < nrows; ++r) {
        int64_t i = rows ? rows[r] : r;
        double *y = Y + r * (int64_t)dim, *ya = Yabs + r * (int64_t)dim;
        for (int32_t c = 0; c < dim; ++c) y[c] = ya[c] = 0.0;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            const float *h = H + (int64_t)col[p] * dim;
            double a = (double)val[p];
            for (int32_t c = 0; c < dim; ++c) {
                double term = a * (double)h[c];
                y[c] += term;
                ya[c] += fabs(term);
            }
        }
    }
    return 0;
}

/* --------------------------------------------------------------- backward */

/*
 * Outer product, sampled (Eq. 3, Alg. 2):  for every stored entry (i, j=col[p]):
 *     D[j,t] += val[p] * dY[i, sp_index[j,t]]      for t in [0,k)
 * i.e. D = (A^T dY) read at each row's CBSR columns.  Written as the plain
 * scatter over the CSR rows of A; no transposed structure is built.
 * slot == NULL: D, Dabs are N x k.  Otherwise slot[j] is the output row of
 * node j, or -1 to skip it, and D, Dabs have nslots x k entries.
 * src_begin/src_end restrict the source rows i (whole matrix: 0, N); that
 * restriction exists only so a timed sample can be bounded.
 */
int oracle_sspmm_bwd(int64_t N, const int32_t *rowptr, const int32_t *col, const float *val, const float *dY,
                     const int32_t *sp_index, int32_t dim, int32_t k, const int64_t *slot, int64_t nslots,
                     int64_t src_begin, int64_t src_end, double *D, double *Dabs)
{
    if (N < 0 || dim < 1 || k < 1 || k > dim) return -1;
    if (!slot) nslots = N;
    memset(D, 0, sizeof(double) * (size_t)(nslots * k));
    memset(Dabs, 0, sizeof(double) * (size_t)(nslots * k));
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = src_begin; i < src_end; ++i) {
        const float *g = dY + i * (int64_t)dim;
        for (int64_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int64_t j = col[p];
            int64_t o = slot ? slot[j] : j;
            if (o < 0) continue;
            double a = (double)val[p];
            const int32_t *ix = sp_index + j * k;
            for (int32_t t = 0; t < k; ++t) {
                double term = a * (double)g[ix[t]];
                double at = fabs(term);
#pragma omp atomic
                D[o * k + t] += term;
#pragma omp atomic
                Dabs[o * k + t] += at;
            }
        }
    }
    return 0;
}

/*
 * MaxK backward (Sec. 3.1 definition, part (ii): the gradient keeps the forward sparsity pattern):
 * dH[i, sp_index[i,t]] = dXs[i,t], every other entry of dH is zero.  Pure placement, no arithmetic.
 */
int oracle_cbsr_scatter(const float *dXs, const int32_t *sp_index, int64_t N, int32_t dim, int32_t k, float *dH)
{
    if (N < 0 || dim < 1 || k < 1 || k > dim) return -1;
    memset(dH, 0, sizeof(float) * (size_t)(N * dim));
    for (int64_t i = 0; i < N; ++i)
        for (int32_t t = 0; t < k; ++t) dH[i * (int64_t)dim + sp_index[i * (int64_t)k + t]] = dXs[i * (int64_t)k + t];
    return 0;
}

int32_t oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
