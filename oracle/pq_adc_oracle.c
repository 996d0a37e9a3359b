/*
 * CPU oracle for product-quantised asymmetric distance computation (ADC).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow definition that the
 * GPU library's results are compared with.  It shares no code with the
 * library, is never linked into it, and nothing in the product path may call
 * it.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
 * load it.
 *
 * Everything here is written straight from the paper's statement of the
 * problem (sections "Introduction" and "Related Work", Eq. 1):
 *   - a d-dimensional vector is split into M contiguous groups of ds = d/M
 *     dimensions; group m has a codebook of K codewords of ds dimensions;
 *   - a vector is encoded by the index of the nearest codeword in each group;
 *   - the distance between an uncompressed query q and an encoded vector is
 *     the sum over the M groups of the precomputed table entry
 *     ||q^(m) - c_m(i_m)||^2  ("M table lookups and M-1 additions").
 * Reading taken where Eq. 1 is ambiguous: the table is defined on the ds
 * dimensions of each group only (not on zero-padded full-length codewords), so
 * the second and third terms of Eq. 1 vanish and the sum equals the squared
 * Euclidean distance to the reconstructed vector exactly.  Distances are
 * squared L2; codes are 0-based.
 *
 * The encoding tree and forest of the paper are re-associations of the same
 * sum, so they have no separate definition here: the flat sum is the truth for
 * every mode.
 *
 * Arithmetic: inputs are float32 values widened to double; every accumulation
 * is in double.  Loops are in the order of the definition: no blocking, no
 * SIMD intrinsics.  OpenMP, when enabled, splits only the outermost loop over
 * independent vectors or queries.
 *
 * Pins (tests/test_oracle_*.py): brute-force distance to decoded vectors,
 * nearest-codeword optimality by exhaustive search, the lossless-quantiser
 * special case against a library pairwise-distance routine, M=1 / K=1 /
 * query-equals-reconstruction special cases, a hand-worked example stored
 * under tests/golden/, and top-k against a library lexicographic sort.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <float.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ENOMEM (-2)

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static int check_shape(int d, int M, int K)
{
    if (d <= 0 || M <= 0 || K <= 0 || K > 256) return ORC_EINVAL;
    if (d % M != 0) return ORC_EINVAL;
    return ORC_OK;
}

/* squared L2 distance between a float sub-vector and a double codeword */
static double sqdist_fd(const float *a, const double *b, int n)
{
    double s = 0.0;
    for (int j = 0; j < n; ++j) {
        double t = (double)a[j] - b[j];
        s += t * t;
    }
    return s;
}

/* squared L2 distance between two float sub-vectors, in double */
static double sqdist_ff(const float *a, const float *b, int n)
{
    double s = 0.0;
    for (int j = 0; j < n; ++j) {
        double t = (double)a[j] - (double)b[j];
        s += t * t;
    }
    return s;
}

/*
 * Lloyd's k-means, one independent run per dimension group ("quantize each
 * dimension group separately", Introduction).
 *   x          [n][d] training vectors
 *   init_rows  [M][K] row numbers of x whose group-m sub-vector is the initial
 *              codeword k of group m (the random draw is the caller's input)
 *   codebooks  [M][K][ds] out, float32 (rounded once, after the last update)
 *   objective  [M][iters] out (may be NULL): mean squared quantisation error of
 *              group m measured in the assignment step of iteration it, i.e.
 *              with the centroids that iteration started from
 * Assignment: nearest centroid, lowest index on ties.  Update: arithmetic mean
 * of the assigned sub-vectors; a centroid with no assigned vector keeps its
 * previous value.
 */
int orc_kmeans(const float *x, int64_t n, int d, int M, int K, int iters,
               const int64_t *init_rows, float *codebooks, double *objective)
{
    int rc = check_shape(d, M, K);
    if (rc) return rc;
    if (!x || !init_rows || !codebooks || n <= 0 || iters < 0) return ORC_EINVAL;
    const int ds = d / M;
    double *cent = (double *)malloc(sizeof(double) * (size_t)K * ds);
    double *sum = (double *)malloc(sizeof(double) * (size_t)K * ds);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)K);
    int *assign = (int *)malloc(sizeof(int) * (size_t)n);
    if (!cent || !sum || !cnt || !assign) {
        free(cent); free(sum); free(cnt); free(assign);
        return ORC_ENOMEM;
    }
    for (int m = 0; m < M; ++m) {
        for (int k = 0; k < K; ++k) {
            int64_t r = init_rows[(size_t)m * K + k];
            if (r < 0 || r >= n) { free(cent); free(sum); free(cnt); free(assign); return ORC_EINVAL; }
            for (int j = 0; j < ds; ++j)
                cent[(size_t)k * ds + j] = (double)x[(size_t)r * d + (size_t)m * ds + j];
        }
        for (int it = 0; it < iters; ++it) {
            double obj = 0.0;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) reduction(+ : obj)
#endif
            for (int64_t i = 0; i < n; ++i) {
                const float *xi = x + (size_t)i * d + (size_t)m * ds;
                int best = 0;
                double bestd = DBL_MAX;
                for (int k = 0; k < K; ++k) {
                    double dk = sqdist_fd(xi, cent + (size_t)k * ds, ds);
                    if (dk < bestd) { bestd = dk; best = k; }
                }
                assign[i] = best;
                obj += bestd;
            }
            if (objective) objective[(size_t)m * iters + it] = obj / (double)n;
            memset(sum, 0, sizeof(double) * (size_t)K * ds);
            memset(cnt, 0, sizeof(int64_t) * (size_t)K);
            for (int64_t i = 0; i < n; ++i) {
                const float *xi = x + (size_t)i * d + (size_t)m * ds;
                int k = assign[i];
                cnt[k] += 1;
                for (int j = 0; j < ds; ++j) sum[(size_t)k * ds + j] += (double)xi[j];
            }
            for (int k = 0; k < K; ++k) {
                if (cnt[k] == 0) continue;
                for (int j = 0; j < ds; ++j)
                    cent[(size_t)k * ds + j] = sum[(size_t)k * ds + j] / (double)cnt[k];
            }
        }
        for (int k = 0; k < K; ++k)
            for (int j = 0; j < ds; ++j)
                codebooks[((size_t)m * K + k) * ds + j] = (float)cent[(size_t)k * ds + j];
    }
    free(cent); free(sum); free(cnt); free(assign);
    return ORC_OK;
}

/*
 * Encoding (Related Work: "encode a vector x with C_m on the corresponding
 * dimensions"): codes[i][m] = argmin_k ||x_i^(m) - c_m(k)||^2, lowest k on ties.
 */
int orc_encode(const float *x, int64_t n, int d, int M, int K,
               const float *codebooks, uint8_t *codes)
{
    int rc = check_shape(d, M, K);
    if (rc) return rc;
    if ((!x && n > 0) || !codebooks || (!codes && n > 0) || n < 0) return ORC_EINVAL;
    const int ds = d / M;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < n; ++i) {
        for (int m = 0; m < M; ++m) {
            const float *xi = x + (size_t)i * d + (size_t)m * ds;
            int best = 0;
            double bestd = DBL_MAX;
            for (int k = 0; k < K; ++k) {
                double dk = sqdist_ff(xi, codebooks + ((size_t)m * K + k) * ds, ds);
                if (dk < bestd) { bestd = dk; best = k; }
            }
            codes[(size_t)i * M + m] = (uint8_t)best;
        }
    }
    return ORC_OK;
}

/*
 * The same quantiser decided in single precision: every squared distance is
 * the float32 sum of float32 products, terms added in index order, each
 * operation rounded on its own (no fused multiply-add), lowest index on ties.
 * This is the arithmetic a float32 encoder can reproduce bit for bit; it is
 * the reference for encoders that work in float32 (the paper fixes no
 * precision for the assignment step).
 */
int orc_encode_f32(const float *x, int64_t n, int d, int M, int K,
                   const float *codebooks, uint8_t *codes)
{
    int rc = check_shape(d, M, K);
    if (rc) return rc;
    if ((!x && n > 0) || !codebooks || (!codes && n > 0) || n < 0) return ORC_EINVAL;
    const int ds = d / M;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < n; ++i) {
        for (int m = 0; m < M; ++m) {
            const float *xi = x + (size_t)i * d + (size_t)m * ds;
            int best = 0;
            float bestd = FLT_MAX;
            for (int k = 0; k < K; ++k) {
                const float *c = codebooks + ((size_t)m * K + k) * ds;
                volatile float s = 0.0f;     /* volatile: one rounding per operation, no contraction */
                for (int j = 0; j < ds; ++j) {
                    volatile float t = xi[j] - c[j];
                    volatile float t2 = t * t;
                    s = s + t2;
                }
                if (s < bestd) { bestd = s; best = k; }
            }
            codes[(size_t)i * M + m] = (uint8_t)best;
        }
    }
    return ORC_OK;
}

/*
 * Reconstruction (Introduction: "approximated by the concatenation of M
 * codewords assigned"): xhat[i] = [c_1(i_1) | c_2(i_2) | ... | c_M(i_M)].
 */
int orc_decode(const uint8_t *codes, int64_t n, int d, int M, int K,
               const float *codebooks, double *xhat)
{
    int rc = check_shape(d, M, K);
    if (rc) return rc;
    if ((!codes && n > 0) || !codebooks || (!xhat && n > 0) || n < 0) return ORC_EINVAL;
    const int ds = d / M;
    for (int64_t i = 0; i < n; ++i)
        for (int m = 0; m < M; ++m) {
            int k = codes[(size_t)i * M + m];
            if (k >= K) return ORC_EINVAL;
            for (int j = 0; j < ds; ++j)
                xhat[(size_t)i * d + (size_t)m * ds + j] =
                    (double)codebooks[((size_t)m * K + k) * ds + j];
        }
    return ORC_OK;
}

/* Exact squared distance between one query and n full-length vectors. */
int orc_brute(const float *q, const double *xhat, int64_t n, int d, double *out)
{
    if (!q || (!xhat && n > 0) || (!out && n > 0) || n < 0 || d <= 0) return ORC_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int j = 0; j < d; ++j) {
            double t = (double)q[j] - xhat[(size_t)i * d + j];
            s += t * t;
        }
        out[i] = s;
    }
    return ORC_OK;
}

/*
 * Precomputed distance table of one query (first term of Eq. 1, restricted to
 * each group's own dimensions): lut[m][k] = ||q^(m) - c_m(k)||^2.
 */
int orc_lut(const float *q, int d, int M, int K, const float *codebooks, double *lut)
{
    int rc = check_shape(d, M, K);
    if (rc) return rc;
    if (!q || !codebooks || !lut) return ORC_EINVAL;
    const int ds = d / M;
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < K; ++k)
            lut[(size_t)m * K + k] =
                sqdist_ff(q + (size_t)m * ds, codebooks + ((size_t)m * K + k) * ds, ds);
    return ORC_OK;
}

/*
 * Flat ADC of one query: dist[n] = lut[0][code[n][0]] + ... + lut[M-1][code[n][M-1]],
 * added left to right.
 */
int orc_adc_flat(const double *lut, const uint8_t *codes, int64_t N, int M, int K, double *dist)
{
    if (!lut || (!codes && N > 0) || (!dist && N > 0) || N < 0 || M <= 0 || K <= 0 || K > 256)
        return ORC_EINVAL;
    for (int64_t n = 0; n < N; ++n) {
        double s = 0.0;
        for (int m = 0; m < M; ++m) {
            int k = codes[(size_t)n * M + m];
            if (k >= K) return ORC_EINVAL;
            s += lut[(size_t)m * K + k];
        }
        dist[n] = s;
    }
    return ORC_OK;
}

typedef struct { double d; int32_t id; } orc_pair;

static int pair_cmp(const void *a, const void *b)
{
    const orc_pair *x = (const orc_pair *)a, *y = (const orc_pair *)b;
    if (x->d < y->d) return -1;
    if (x->d > y->d) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}

/*
 * Top-k by full sort: order all N (distance, id) pairs ascending by distance,
 * ties by smaller id, and return the first k.  ids == NULL means id n = n.
 * (The paper has no selection step; this is the plain definition of "the k
 * nearest encodings" used by the benchmark configurations.)
 */
int orc_topk(const double *dist, const int32_t *ids, int64_t N, int k,
             int32_t *out_ids, double *out_dist)
{
    if ((!dist && N > 0) || k < 0 || k > N || (k > 0 && (!out_ids || !out_dist))) return ORC_EINVAL;
    orc_pair *p = (orc_pair *)malloc(sizeof(orc_pair) * (size_t)(N > 0 ? N : 1));
    if (!p) return ORC_ENOMEM;
    for (int64_t n = 0; n < N; ++n) { p[n].d = dist[n]; p[n].id = ids ? ids[n] : (int32_t)n; }
    qsort(p, (size_t)N, sizeof(orc_pair), pair_cmp);
    for (int i = 0; i < k; ++i) { out_ids[i] = p[i].id; out_dist[i] = p[i].d; }
    free(p);
    return ORC_OK;
}

/*
 * All-pairs ADC: dist[q][n] for Q queries (table, then flat sum, per query).
 */
int orc_adc_all(const float *queries, int64_t Q, int d, int M, int K, const float *codebooks,
                const uint8_t *codes, int64_t N, double *dist)
{
    int rc = check_shape(d, M, K);
    if (rc) return rc;
    if ((!queries && Q > 0) || !codebooks || (!codes && N > 0) || (!dist && Q * N > 0)) return ORC_EINVAL;
    int fail = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int64_t qi = 0; qi < Q; ++qi) {
        double *lut = (double *)malloc(sizeof(double) * (size_t)M * K);
        if (!lut) { fail = ORC_ENOMEM; continue; }
        int r = orc_lut(queries + (size_t)qi * d, d, M, K, codebooks, lut);
        if (!r) r = orc_adc_flat(lut, codes, N, M, K, dist + (size_t)qi * N);
        if (r) fail = r;
        free(lut);
    }
    return fail;
}

/*
 * Search: per query, table -> flat ADC over all N encodings -> top-k by full sort.
 * out_ids [Q][k], out_dist [Q][k].
 */
int orc_search(const float *queries, int64_t Q, int d, int M, int K, const float *codebooks,
               const uint8_t *codes, const int32_t *ids, int64_t N, int k,
               int32_t *out_ids, double *out_dist)
{
    int rc = check_shape(d, M, K);
    if (rc) return rc;
    if ((!queries && Q > 0) || !codebooks || (!codes && N > 0) || k < 0 || k > N) return ORC_EINVAL;
    int fail = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int64_t qi = 0; qi < Q; ++qi) {
        double *lut = (double *)malloc(sizeof(double) * (size_t)M * K);
        double *dist = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        int r = ORC_OK;
        if (!lut || !dist) r = ORC_ENOMEM;
        if (!r) r = orc_lut(queries + (size_t)qi * d, d, M, K, codebooks, lut);
        if (!r) r = orc_adc_flat(lut, codes, N, M, K, dist);
        if (!r) r = orc_topk(dist, ids, N, k, out_ids + (size_t)qi * k, out_dist + (size_t)qi * k);
        if (r) fail = r;
        free(lut); free(dist);
    }
    return fail;
}
