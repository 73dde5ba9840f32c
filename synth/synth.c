/*
 * Seeded synthetic inputs for the MaxK-GNN aggregation path: graphs (uniform
 * and R-MAT, deduplicated, optionally symmetrised, self-loops added, CSR with
 * sorted unique columns), GCN edge weights, and feature matrices.
 *
 * This file holds NONE of the method's arithmetic (no top-k, no aggregation).
 * It only manufactures inputs; the same arrays are handed to the CPU oracle
 * and to the HIP library.  Every random number is a pure function of
 * (seed, stream, counter), so results do not depend on the thread count.
 *
 * Plain C + OpenMP.  Build: gcc -O2 -fopenmp -shared -fPIC synth.c -o libsynth.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---------------------------------------------------------------- RNG -- */

static inline uint64_t mix64(uint64_t z)
{
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* counter-based: one 64-bit word per (seed, stream, counter) */
static inline uint64_t rnd64(uint64_t seed, uint64_t stream, uint64_t ctr)
{
    return mix64(mix64(seed * 0xD1342543DE82EF95ull + stream) ^ (ctr * 0xA0761D6478BD642Full + 1));
}

static inline double u01(uint64_t w) /* (0,1] */
{
    return ((double)(w >> 11) + 1.0) * (1.0 / 9007199254740992.0);
}

/* one standard normal per counter (Box-Muller on two hashed uniforms, fp64) */
static inline double normal_at(uint64_t seed, uint64_t stream, uint64_t ctr)
{
    double u1 = u01(rnd64(seed, stream, 2 * ctr));
    double u2 = u01(rnd64(seed, stream, 2 * ctr + 1));
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
}

enum { STREAM_FEAT = 1, STREAM_EDGE = 2, STREAM_PERM = 3, STREAM_TIEROW = 4, STREAM_POOL = 5, STREAM_PICK = 6 };

/* ----------------------------------------------------------- features -- */

/* out[i] = fp32(N(0,1)) for i in [0,n) */
void synth_normal_f32(uint64_t seed, int64_t n, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) out[i] = (float)normal_at(seed, STREAM_FEAT, (uint64_t)i);
}

/*
 * Overwrite a fraction of the rows of an N x dim matrix with "tie rows":
 * every entry drawn with replacement from a per-row pool of `pool` distinct
 * normals, so equal values straddle any rank; one tie row in `const_every`
 * is constant 0.0f.  Row choice is a hash of the row id.  Returns the number
 * of rows rewritten.
 */
int64_t synth_tie_rows(uint64_t seed, int64_t N, int32_t dim, int32_t percent, int32_t pool, int32_t const_every,
                       float *H)
{
    int64_t count = 0;
    if (pool > 256) pool = 256;
#pragma omp parallel for schedule(static) reduction(+ : count)
    for (int64_t i = 0; i < N; ++i) {
        uint64_t h = rnd64(seed, STREAM_TIEROW, (uint64_t)i);
        if ((int32_t)(h % 100u) >= percent) continue;
        ++count;
        float *row = H + i * (int64_t)dim;
        if (const_every > 0 && ((h >> 32) % (uint64_t)const_every) == 0) {
            for (int32_t c = 0; c < dim; ++c) row[c] = 0.0f;
            continue;
        }
        float pv[256];
        for (int32_t j = 0; j < pool; ++j) pv[j] = (float)normal_at(seed, STREAM_POOL, (uint64_t)i * 256u + (uint64_t)j);
        for (int32_t c = 0; c < dim; ++c) {
            uint64_t r = rnd64(seed, STREAM_PICK, (uint64_t)i * (uint64_t)dim + (uint64_t)c);
            row[c] = pv[r % (uint64_t)pool];
        }
    }
    return count;
}

/* ----------------------------------------------------- parallel radix -- */

#define RADIX_BITS 11
#define RADIX_SIZE (1 << RADIX_BITS)

/* stable LSD radix sort of 64-bit keys (low `bits` bits significant) with an
 * optional 32-bit payload; tmp buffers must hold n elements. */
static void radix_sort_u64(uint64_t *keys, uint32_t *pay, uint64_t *tkeys, uint32_t *tpay, int64_t n, int bits)
{
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    int64_t *hist = (int64_t *)malloc(sizeof(int64_t) * (size_t)nthreads * RADIX_SIZE);
    uint64_t *src = keys, *dst = tkeys;
    uint32_t *psrc = pay, *pdst = tpay;
    for (int shift = 0; shift < bits; shift += RADIX_BITS) {
#pragma omp parallel num_threads(nthreads)
        {
            int tid = 0, nt = 1;
#ifdef _OPENMP
            tid = omp_get_thread_num();
            nt = omp_get_num_threads(); /* may be fewer than requested */
#endif
            int64_t lo = n * tid / nt, hi = n * (tid + 1) / nt;
            int64_t *h = hist + (size_t)tid * RADIX_SIZE;
            memset(h, 0, sizeof(int64_t) * RADIX_SIZE);
            for (int64_t i = lo; i < hi; ++i) ++h[(src[i] >> shift) & (RADIX_SIZE - 1)];
#pragma omp barrier
#pragma omp single
            {
                int64_t run = 0;
                for (int d = 0; d < RADIX_SIZE; ++d)
                    for (int t = 0; t < nt; ++t) {
                        int64_t c = hist[(size_t)t * RADIX_SIZE + d];
                        hist[(size_t)t * RADIX_SIZE + d] = run;
                        run += c;
                    }
            }
            if (psrc) {
                for (int64_t i = lo; i < hi; ++i) {
                    int64_t p = h[(src[i] >> shift) & (RADIX_SIZE - 1)]++;
                    dst[p] = src[i];
                    pdst[p] = psrc[i];
                }
            } else {
                for (int64_t i = lo; i < hi; ++i) dst[h[(src[i] >> shift) & (RADIX_SIZE - 1)]++] = src[i];
            }
        }
        uint64_t *t = src; src = dst; dst = t;
        uint32_t *pt = psrc; psrc = pdst; pdst = pt;
    }
    if (src != keys) {
        memcpy(keys, src, sizeof(uint64_t) * (size_t)n);
        if (pay) memcpy(pay, psrc, sizeof(uint32_t) * (size_t)n);
    }
    free(hist);
}

static int bits_for(int64_t n)
{
    int b = 1;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

/* -------------------------------------------------------------- edges -- */

/* candidate edge number t -> (u,v) in [0,2^scale)^2 by R-MAT quadrant descent,
 * or uniform over [0,N)^2 when scale == 0 */
static inline void candidate(uint64_t seed, uint64_t t, int scale, int64_t N, uint32_t ta, uint32_t tb, uint32_t tc,
                             int64_t *pu, int64_t *pv)
{
    if (scale == 0) {
        *pu = (int64_t)(rnd64(seed, STREAM_EDGE, 2 * t) % (uint64_t)N);
        *pv = (int64_t)(rnd64(seed, STREAM_EDGE, 2 * t + 1) % (uint64_t)N);
        return;
    }
    int64_t u = 0, v = 0;
    uint64_t w = 0;
    for (int l = 0; l < scale; ++l) {
        if ((l & 1) == 0) w = rnd64(seed, STREAM_EDGE, t * 16 + (uint64_t)(l >> 1));
        uint32_t r = (uint32_t)(w >> ((l & 1) * 32));
        int ub, vb;
        if (r < ta) { ub = 0; vb = 0; }
        else if (r < tb) { ub = 0; vb = 1; }
        else if (r < tc) { ub = 1; vb = 0; }
        else { ub = 1; vb = 1; }
        u = (u << 1) | ub;
        v = (v << 1) | vb;
    }
    *pu = u;
    *pv = v;
}

/*
 * First M unique edges of the candidate stream t = 0,1,2,...
 *   scale  : R-MAT levels (0 = uniform pairs over [0,N))
 *   a,b,c  : R-MAT quadrant probabilities (d = 1-a-b-c)
 *   directed: 0 -> unordered pairs {u,v} (stored u<v), 1 -> ordered pairs
 * Candidates with an endpoint >= N or u == v are skipped.  Endpoints are
 * relabelled by a seeded random permutation so hubs are not contiguous.
 * out_keys[M] receives (u << 32 | v), sorted ascending.
 * Returns the number of candidates consumed, or -1 on failure.
 */
int64_t synth_unique_edges(uint64_t seed, int32_t scale, int64_t N, double a, double b, double c, int64_t M,
                           int32_t directed, uint64_t *out_keys)
{
    if (N < 2 || M < 0 || scale > 31) return -1;
    if (M == 0) return 0;
    uint32_t ta = (uint32_t)(a * 4294967296.0), tb = (uint32_t)((a + b) * 4294967296.0),
             tc = (uint32_t)((a + b + c) * 4294967296.0);
    int nb = bits_for(N);

    /* seeded permutation (Fisher-Yates, serial) */
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    for (int64_t i = 0; i < N; ++i) perm[i] = (int32_t)i;
    for (int64_t i = N - 1; i > 0; --i) {
        int64_t j = (int64_t)(rnd64(seed, STREAM_PERM, (uint64_t)i) % (uint64_t)(i + 1));
        int32_t tmp = perm[i]; perm[i] = perm[j]; perm[j] = tmp;
    }

    int64_t T = M + M / 4 + 1024;
    for (int attempt = 0; attempt < 12; ++attempt, T = T + T / 2) {
        if (T > 0xFFFFFFF0ll) break;
        uint64_t *keys = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)T);
        uint64_t *tkeys = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)T);
        uint32_t *idx = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)T);
        uint32_t *tidx = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)T);
        uint8_t *first = (uint8_t *)calloc((size_t)T, 1);
        if (!keys || !tkeys || !idx || !tidx || !first) { free(keys); free(tkeys); free(idx); free(tidx); free(first); free(perm); return -1; }
        const uint64_t INVALID = ((uint64_t)1 << (2 * nb)) - 1 + 1; /* one past any packed valid key */
#pragma omp parallel for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            int64_t u, v;
            candidate(seed, (uint64_t)t, scale, N, ta, tb, tc, &u, &v);
            uint64_t key = INVALID;
            if (u < N && v < N && u != v) {
                int64_t pu = perm[u], pv = perm[v];
                if (!directed && pu > pv) { int64_t s = pu; pu = pv; pv = s; }
                key = ((uint64_t)pu << nb) | (uint64_t)pv;
            }
            keys[t] = key;
            idx[t] = (uint32_t)t;
        }
        radix_sort_u64(keys, idx, tkeys, tidx, T, 2 * nb + 1);
        /* the first element of each run of equal keys has the smallest t (stable sort) */
#pragma omp parallel for schedule(static)
        for (int64_t s = 0; s < T; ++s)
            if (keys[s] != INVALID && (s == 0 || keys[s - 1] != keys[s])) first[idx[s]] = 1;
        int64_t seen = 0, tstar = -1;
        for (int64_t t = 0; t < T; ++t) {
            seen += first[t];
            if (seen == M) { tstar = t; break; }
        }
        if (tstar >= 0) {
            int64_t w = 0;
            for (int64_t s = 0; s < T; ++s)
                if (keys[s] != INVALID && (s == 0 || keys[s - 1] != keys[s]) && (int64_t)idx[s] <= tstar) {
                    uint64_t pu = keys[s] >> nb, pv = keys[s] & (((uint64_t)1 << nb) - 1);
                    out_keys[w++] = (pu << 32) | pv;
                }
            free(keys); free(tkeys); free(idx); free(tidx); free(first); free(perm);
            return (w == M) ? tstar + 1 : -1;
        }
        free(keys); free(tkeys); free(idx); free(tidx); free(first);
    }
    free(perm);
    return -1;
}

/*
 * CSR from M unique edges (u << 32 | v, u != v).
 *   symmetrise: also store (v,u) for every (u,v)
 *   self_loops: also store (i,i) for every i
 * rowptr[N+1], col[nnz] with nnz = M*(symmetrise?2:1) + (self_loops?N:0);
 * columns sorted ascending and unique within each row.  Returns nnz or -1.
 */
int64_t synth_build_csr(const uint64_t *edge_keys, int64_t M, int64_t N, int32_t symmetrise, int32_t self_loops,
                        int32_t *rowptr, int32_t *col)
{
    int64_t nnz = M * (symmetrise ? 2 : 1) + (self_loops ? N : 0);
    if (nnz > 0x7FFFFFF0ll) return -1;
    int nb = bits_for(N);
    uint64_t *keys = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)(nnz > 0 ? nnz : 1));
    uint64_t *tmp = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)(nnz > 0 ? nnz : 1));
    if (!keys || !tmp) { free(keys); free(tmp); return -1; }
    const uint64_t lowmask = 0xFFFFFFFFull;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < M; ++e) {
        uint64_t u = edge_keys[e] >> 32, v = edge_keys[e] & lowmask;
        if (symmetrise) {
            keys[2 * e] = (u << nb) | v;
            keys[2 * e + 1] = (v << nb) | u;
        } else {
            keys[e] = (u << nb) | v;
        }
    }
    int64_t base = M * (symmetrise ? 2 : 1);
    if (self_loops)
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; ++i) keys[base + i] = ((uint64_t)i << nb) | (uint64_t)i;
    radix_sort_u64(keys, NULL, tmp, NULL, nnz, 2 * nb);
    memset(rowptr, 0, sizeof(int32_t) * (size_t)(N + 1));
    const uint64_t cmask = ((uint64_t)1 << nb) - 1;
    for (int64_t p = 0; p < nnz; ++p) ++rowptr[(keys[p] >> nb) + 1];
    for (int64_t i = 0; i < N; ++i) rowptr[i + 1] += rowptr[i];
#pragma omp parallel for schedule(static)
    for (int64_t p = 0; p < nnz; ++p) col[p] = (int32_t)(keys[p] & cmask);
    free(keys);
    free(tmp);
    return nnz;
}

/* GCN-style weights: val[p] = fp32( 1/sqrt(d_i * d_j) ), d = stored entries of the row */
void synth_gcn_weights(int64_t N, const int32_t *rowptr, const int32_t *col, float *val)
{
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t i = 0; i < N; ++i) {
        double di = (double)(rowptr[i + 1] - rowptr[i]);
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int32_t j = col[p];
            double dj = (double)(rowptr[j + 1] - rowptr[j]);
            if (dj < 1.0) dj = 1.0; /* node with no stored out-entries (directed graphs without self-loops) */
            val[p] = (float)(1.0 / sqrt(di * dj));
        }
    }
}

/* mean-aggregator weights (GraphSAGE): val[p] = fp32(1/d_i) -- a non-symmetric matrix */
void synth_mean_weights(int64_t N, const int32_t *rowptr, float *val)
{
#pragma omp parallel for schedule(dynamic, 1024)
    for (int64_t i = 0; i < N; ++i) {
        double di = (double)(rowptr[i + 1] - rowptr[i]);
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) val[p] = (float)(1.0 / di);
    }
}

int32_t synth_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
