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
 *   oracle_narrow / oracle_widen   fp32 <-> 16-bit CBSR values (bf16, fp16), round to nearest even:
 *                      the sp_data term of the forward traffic model, Sec. 4.3, stored in 2 bytes
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
 * non-symmetric matrix, NumPy stable argsort, hand-worked goldens; the 16-bit
 * conversions against NumPy's float16 and PyTorch's bfloat16 casts, hand-worked
 * halfway cases, and the round trip over all 65536 bit patterns.
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

/* ------------------------------------------------- 16-bit CBSR values */

/*
 * Narrow CBSR values (the sp_data array of Sec. 3.2, whose bytes per entry enter the forward
 * traffic model of Sec. 4.3).  type 1 = bfloat16 (1 sign, 8 exponent, 7 fraction bits),
 * type 2 = IEEE binary16 (1, 5, 10; subnormals kept).  Rounding: to nearest, halfway cases to
 * the even neighbour; magnitudes beyond the largest finite value round to infinity as IEEE
 * prescribes.  NaN is outside the contract (returns -1).
 */
static int narrow_bf16(float x, uint16_t *out)
{
    uint32_t b;
    memcpy(&b, &x, 4);
    if (x != x) return -1;
    /* For one sign, fp32 bit patterns grow with magnitude, and bf16 is fp32 with the low 16 bits cut:
     * the two bf16 neighbours of x are the pattern with those bits cleared and the next one up. */
    uint32_t below = b >> 16, rest = b & 0xFFFFu;
    uint32_t above = below + 1u;  /* carries into the exponent (up to infinity) exactly as the value grows */
    if (rest > 0x8000u) *out = (uint16_t)above;
    else if (rest < 0x8000u) *out = (uint16_t)below;
    else *out = (uint16_t)((below & 1u) ? above : below);  /* halfway: the neighbour with an even last bit */
    return 0;
}

static int narrow_f16(float x, uint16_t *out)
{
    if (x != x) return -1;
    const uint16_t sign = signbit(x) ? 0x8000u : 0u;
    double a = fabs((double)x);
    if (isinf(a)) { *out = sign | 0x7C00u; return 0; }
    /* spacing of binary16 values around a: 2^(e-10) for a in [2^e, 2^(e+1)), e >= -14; 2^-24 below 2^-14 */
    int e;
    (void)frexp(a, &e);        /* a = m * 2^e, m in [0.5, 1)  ->  a in [2^(e-1), 2^e) */
    e -= 1;
    if (a == 0.0 || e < -14) e = -14;
    const double quantum = ldexp(1.0, e - 10);
    const double q = nearbyint(a / quantum);   /* default rounding mode: nearest, ties to even; a/quantum is exact */
    const double r = q * quantum;              /* the rounded magnitude, exact */
    if (r >= 65536.0) { *out = sign | 0x7C00u; return 0; }  /* past the largest finite value 65504 */
    if (r == 0.0) { *out = sign; return 0; }
    if (r < ldexp(1.0, -14)) { *out = sign | (uint16_t)(r / ldexp(1.0, -24)); return 0; }  /* subnormal: fraction counts 2^-24 */
    int er;
    const double m = frexp(r, &er);            /* r = m * 2^er, m in [0.5, 1) */
    const int biased = (er - 1) + 15;
    const uint16_t frac = (uint16_t)((m * 2.0 - 1.0) * 1024.0);
    *out = sign | (uint16_t)(biased << 10) | frac;
    return 0;
}

int oracle_narrow(const float *x, int64_t n, int32_t type, uint16_t *out)
{
    if (type != 1 && type != 2) return -1;
    int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
    for (int64_t i = 0; i < n; ++i) bad |= (type == 1 ? narrow_bf16(x[i], &out[i]) : narrow_f16(x[i], &out[i])) != 0;
    return bad ? -1 : 0;
}

/* The value a 16-bit pattern stands for, as fp32 (exact: both formats are subsets of fp32). */
int oracle_widen(const uint16_t *h, int64_t n, int32_t type, float *out)
{
    if (type != 1 && type != 2) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const uint16_t b = h[i];
        const int neg = b >> 15;
        double v;
        if (type == 1) {
            const int ex = (b >> 7) & 0xFF, fr = b & 0x7F;
            if (ex == 0xFF) v = fr ? NAN : INFINITY;
            else if (ex == 0) v = ldexp((double)fr, -126 - 7);
            else v = ldexp(1.0 + fr / 128.0, ex - 127);
        } else {
            const int ex = (b >> 10) & 0x1F, fr = b & 0x3FF;
            if (ex == 0x1F) v = fr ? NAN : INFINITY;
            else if (ex == 0) v = ldexp((double)fr, -24);
            else v = ldexp(1.0 + fr / 1024.0, ex - 15);
        }
        out[i] = (float)(neg ? -v : v);
    }
    return 0;
}
