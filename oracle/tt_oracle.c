/*
 * CPU oracle for the TT-EmbeddingBag path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously correct implementation of what the hot path
 * computes, written from the paper's definitions.  It is used by the tests,
 * by the smoke check and by the benchmark's cpu_baseline leg, and by nothing
 * else; the product path never calls it.  It shares no code, header, table or
 * helper with the HIP library.
 *
 * Arithmetic: inputs and outputs are fp32 (the paper does not fix a precision;
 * the cores are fp32 parameters), every product and sum is carried in fp64 and
 * each result element is rounded to fp32 once, at the end.
 *
 * Storage convention used here: core k is a C array
 *     G_k[m_k][r_{k-1}][n_k][r_k]
 * i.e. the paper's 4-way core G_k in R^{r_{k-1} x m_k x n_k x r_k} (Section 2,
 * Eq. 2) with the row digit moved to the front, so that the slice picked by a
 * digit is one contiguous block.  d = 3 throughout (Alg. 1 and 2 are printed
 * for the 3-core case).
 *
 * Every function is pinned by tests/test_oracle_*.py against something other
 * than itself (Table 1's parameter counts, dense reconstruction with a library
 * einsum, library embedding_bag + autograd, finite differences, closed forms).
 * The Zipf sampler and the core initialisation live in the workload generator,
 * not here, and are "parity unpinned" harness conventions.
 */

#ifdef _OPENMP
#include <omp.h>
#endif
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- shape arithmetic --------------------------------------------------- */

/* Number of parameters of the three cores: sum_k r_{k-1} m_k n_k r_k
 * (Section 2, Eq. 2; the "# of TT Parameters" columns of Table 1). */
int64_t ora_param_count(const int64_t m[3], const int64_t n[3], const int64_t r[4])
{
    int64_t total = 0;
    for (int k = 0; k < 3; ++k)
        total += r[k] * m[k] * n[k] * r[k + 1];
    return total;
}

/* ---- digits ------------------------------------------------------------- */

/* Row index -> mixed-radix digits, i = i1*m2*m3 + i2*m3 + i3 with i1 the most
 * significant digit (Section 3.1, the sentence before Eq. 3, read with the sum
 * running over k). */
void ora_decode(const int64_t m[3], const int64_t *indices, int64_t L,
                int32_t *i1, int32_t *i2, int32_t *i3)
{
    for (int64_t k = 0; k < L; ++k) {
        int64_t i = indices[k];
        i3[k] = (int32_t)(i % m[2]);
        i2[k] = (int32_t)((i / m[2]) % m[1]);
        i1[k] = (int32_t)(i / (m[1] * m[2]));
    }
}

/* ---- one row ------------------------------------------------------------ */

/* Eq. 3: w_i(j1,j2,j3) = sum_a sum_b G1[i1][0][j1][a] G2[i2][a][j2][b] G3[i3][b][j3][0],
 * written out element by element.  Output column j = (j1*n2 + j2)*n3 + j3
 * (row-major unfolding of Section 3.1's partial products). */
void ora_row(const int64_t m[3], const int64_t n[3], const int64_t r[4],
             const float *G1, const float *G2, const float *G3,
             int64_t row_id, double *out)
{
    const int64_t R1 = r[1], R2 = r[2];
    const int64_t i3 = row_id % m[2];
    const int64_t i2 = (row_id / m[2]) % m[1];
    const int64_t i1 = row_id / (m[1] * m[2]);
    const float *A = G1 + i1 * (n[0] * R1);             /* [n1][R1]          */
    const float *B = G2 + i2 * (R1 * n[1] * R2);        /* [R1][n2][R2]      */
    const float *C = G3 + i3 * (R2 * n[2]);             /* [R2][n3]          */
    for (int64_t j1 = 0; j1 < n[0]; ++j1)
        for (int64_t j2 = 0; j2 < n[1]; ++j2)
            for (int64_t j3 = 0; j3 < n[2]; ++j3) {
                double s = 0.0;
                for (int64_t a = 0; a < R1; ++a)
                    for (int64_t b = 0; b < R2; ++b)
                        s += (double)A[j1 * R1 + a] *
                             (double)B[(a * n[1] + j2) * R2 + b] *
                             (double)C[b * n[2] + j3];
                out[(j1 * n[1] + j2) * n[2] + j3] = s;
            }
}

/* ---- cache -------------------------------------------------------------- */

/* Dense row -> slot map (-1 = not cached).  Obvious, O(num_rows) memory. */
static int32_t *build_slot_map(int64_t num_rows, const int64_t *keys, int64_t K)
{
    int32_t *map = (int32_t *)malloc((size_t)num_rows * sizeof(int32_t));
    if (!map) return NULL;
    for (int64_t i = 0; i < num_rows; ++i) map[i] = -1;
    for (int64_t s = 0; s < K; ++s) map[keys[s]] = (int32_t)s;
    return map;
}

/* slot[k] = position of indices[k] among the cached rows, else -1
 * (Section 4.2: indices are split into cached ones and TT ones). */
int ora_cache_lookup(int64_t num_rows, const int64_t *keys, int64_t K,
                     const int64_t *indices, int64_t L, int32_t *slot)
{
    int32_t *map = build_slot_map(num_rows, keys, K);
    if (!map) return -1;
    for (int64_t k = 0; k < L; ++k) slot[k] = map[indices[k]];
    free(map);
    return 0;
}

typedef struct { int64_t row, count; } cand_t;

static int cand_cmp(const void *pa, const void *pb)
{
    const cand_t *a = (const cand_t *)pa, *b = (const cand_t *)pb;
    if (a->count != b->count) return a->count > b->count ? -1 : 1;   /* most used first   */
    if (a->row != b->row) return a->row < b->row ? -1 : 1;           /* then lower row id */
    return 0;
}

/* Least-frequently-used selection (Section 4.2): the K most frequently used
 * rows are kept.  The paper gives no tie rule; here ties go to the lower row
 * id, and the slot of a row is its rank in that order. */
int ora_cache_select(const int64_t *cand_rows, const int64_t *cand_counts, int64_t n_cand,
                     int64_t K, int64_t *keys)
{
    cand_t *c = (cand_t *)malloc((size_t)(n_cand > 0 ? n_cand : 1) * sizeof(cand_t));
    if (!c) return -1;
    for (int64_t i = 0; i < n_cand; ++i) { c[i].row = cand_rows[i]; c[i].count = cand_counts[i]; }
    qsort(c, (size_t)n_cand, sizeof(cand_t), cand_cmp);
    for (int64_t s = 0; s < K; ++s) keys[s] = c[s].row;
    free(c);
    return 0;
}

/* Cache lines are initialised from the TT cores (Section 4.2): the stored row
 * is the reconstructed row, rounded to fp32. */
void ora_cache_fill(const int64_t m[3], const int64_t n[3], const int64_t r[4],
                    const float *G1, const float *G2, const float *G3,
                    const int64_t *keys, int64_t K, float *rows)
{
    const int64_t N = n[0] * n[1] * n[2];
    double *tmp = (double *)malloc((size_t)N * sizeof(double));
    for (int64_t s = 0; s < K; ++s) {
        ora_row(m, n, r, G1, G2, G3, keys[s], tmp);
        for (int64_t j = 0; j < N; ++j) rows[s * N + j] = (float)tmp[j];
    }
    free(tmp);
}

/* ---- forward ------------------------------------------------------------ */

/* Eq. 5-6 with half-open bags offsets[b] <= k < offsets[b+1] (Section 4.1's
 * prose), sum pooling, optional per-position weight alpha[k] (NULL = 1).
 * A cached row is read from cache_rows instead of being rebuilt (Section 4.2).
 * Lookups are pooled in increasing k.  An empty bag gives a zero row. */
static void fwd_one_bag(const int64_t m[3], const int64_t n[3], const int64_t r[4],
                        const float *G1, const float *G2, const float *G3,
                        const int64_t *indices, const int64_t *offsets, const float *alpha,
                        const int32_t *map, const float *cache_rows,
                        int64_t b, double *acc, double *row, float *output)
{
    const int64_t N = n[0] * n[1] * n[2];
    for (int64_t j = 0; j < N; ++j) acc[j] = 0.0;
    for (int64_t k = offsets[b]; k < offsets[b + 1]; ++k) {
        const int64_t i = indices[k];
        const double w = alpha ? (double)alpha[k] : 1.0;
        if (map && map[i] >= 0) {
            for (int64_t j = 0; j < N; ++j) row[j] = (double)cache_rows[(int64_t)map[i] * N + j];
        } else {
            ora_row(m, n, r, G1, G2, G3, i, row);
        }
        for (int64_t j = 0; j < N; ++j) acc[j] += w * row[j];
    }
    for (int64_t j = 0; j < N; ++j) output[b * N + j] = (float)acc[j];
}

int ora_fwd(const int64_t m[3], const int64_t n[3], const int64_t r[4], int64_t num_rows,
            const float *G1, const float *G2, const float *G3,
            const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
            const float *alpha,
            const int64_t *cache_keys, const float *cache_rows, int64_t K,
            float *output)
{
    const int64_t N = n[0] * n[1] * n[2];
    int32_t *map = NULL;
    (void)L;
    if (K > 0) { map = build_slot_map(num_rows, cache_keys, K); if (!map) return -1; }
    double *acc = (double *)malloc((size_t)N * sizeof(double));
    double *row = (double *)malloc((size_t)N * sizeof(double));
    for (int64_t b = 0; b < n_bags; ++b)
        fwd_one_bag(m, n, r, G1, G2, G3, indices, offsets, alpha, map, cache_rows, b, acc, row, output);
    free(acc); free(row); free(map);
    return 0;
}

/* The same forward pass with the bags shared out among `threads` host threads (a bag is
 * still pooled by one thread, in increasing k, so every output value is the one ora_fwd
 * gives, bit for bit).  Returns the number of threads that ran, or -1.  Only the timing
 * of a multi-core CPU baseline uses it; the tests check it against ora_fwd. */
int ora_fwd_threads(const int64_t m[3], const int64_t n[3], const int64_t r[4], int64_t num_rows,
                    const float *G1, const float *G2, const float *G3,
                    const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
                    const float *alpha,
                    const int64_t *cache_keys, const float *cache_rows, int64_t K,
                    float *output, int threads)
{
    const int64_t N = n[0] * n[1] * n[2];
    int32_t *map = NULL;
    int ran = 1;
    (void)L;
    if (threads < 1) threads = 1;
    if (K > 0) { map = build_slot_map(num_rows, cache_keys, K); if (!map) return -1; }
#pragma omp parallel num_threads(threads)
    {
        double *acc = (double *)malloc((size_t)N * sizeof(double));
        double *row = (double *)malloc((size_t)N * sizeof(double));
#ifdef _OPENMP
#pragma omp single
        ran = omp_get_num_threads();
#endif
#pragma omp for schedule(static)
        for (int64_t b = 0; b < n_bags; ++b)
            fwd_one_bag(m, n, r, G1, G2, G3, indices, offsets, alpha, map, cache_rows, b, acc, row, output);
        free(acc); free(row);
    }
    free(map);
    return ran;
}

/* ---- backward ----------------------------------------------------------- */

/* Gradients of L = <output, grad_output> with respect to the three cores and
 * the cached rows (Section 3.1, Eq. 4 as repaired by ordinary matrix calculus;
 * Alg. 2's wiring computes the same products).  For lookup k in bag b, with
 * dY = alpha_k * grad_output[b] viewed (n1 n2) x n3, A = G1[i1] (n1 x R1),
 * Bm = G2[i2] (R1 x n2 R2), C = G3[i3] (R2 x n3), T0 = A Bm viewed (n1 n2) x R2:
 *     dG3[i3]  += T0^T dY
 *     dT0       = dY C^T
 *     dG2[i2]  += A^T dT0'          (dT0' = dT0 viewed n1 x n2 R2)
 *     dG1[i1]  += dT0' Bm^T
 * A cached lookup contributes dY to dCache[slot] only, and nothing to the cores
 * (the two sets are learned separately, Section 4.2).  Contributions of
 * repeated indices add (Alg. 2, the "+=" line).  The caller provides zeroed
 * fp64 buffers shaped like the cores (and like the cache); this routine adds
 * into them in increasing k. */
int ora_bwd(const int64_t m[3], const int64_t n[3], const int64_t r[4], int64_t num_rows,
            const float *G1, const float *G2, const float *G3,
            const int64_t *indices, int64_t L, const int64_t *offsets, int64_t n_bags,
            const float *alpha,
            const int64_t *cache_keys, int64_t K,
            const float *grad_output,
            double *dG1, double *dG2, double *dG3, double *dCache)
{
    const int64_t n1 = n[0], n2 = n[1], n3 = n[2], R1 = r[1], R2 = r[2];
    const int64_t N = n1 * n2 * n3;
    int32_t *map = NULL;
    (void)L;
    if (K > 0) { map = build_slot_map(num_rows, cache_keys, K); if (!map) return -1; }
    double *T0 = (double *)malloc((size_t)(n1 * n2 * R2) * sizeof(double));
    double *dT0 = (double *)malloc((size_t)(n1 * n2 * R2) * sizeof(double));
    double *dY = (double *)malloc((size_t)N * sizeof(double));
    for (int64_t b = 0; b < n_bags; ++b) {
        for (int64_t k = offsets[b]; k < offsets[b + 1]; ++k) {
            const int64_t i = indices[k];
            const double w = alpha ? (double)alpha[k] : 1.0;
            for (int64_t j = 0; j < N; ++j) dY[j] = w * (double)grad_output[b * N + j];
            if (map && map[i] >= 0) {
                for (int64_t j = 0; j < N; ++j) dCache[(int64_t)map[i] * N + j] += dY[j];
                continue;
            }
            const int64_t i3 = i % m[2];
            const int64_t i2 = (i / m[2]) % m[1];
            const int64_t i1 = i / (m[1] * m[2]);
            const float *A = G1 + i1 * (n1 * R1);
            const float *B = G2 + i2 * (R1 * n2 * R2);
            const float *C = G3 + i3 * (R2 * n3);
            double *gA = dG1 + i1 * (n1 * R1);
            double *gB = dG2 + i2 * (R1 * n2 * R2);
            double *gC = dG3 + i3 * (R2 * n3);
            /* T0[(j1,j2)][b2] = sum_a A[j1][a] Bm[a][(j2,b2)] */
            for (int64_t j1 = 0; j1 < n1; ++j1)
                for (int64_t j2 = 0; j2 < n2; ++j2)
                    for (int64_t b2 = 0; b2 < R2; ++b2) {
                        double s = 0.0;
                        for (int64_t a = 0; a < R1; ++a)
                            s += (double)A[j1 * R1 + a] * (double)B[(a * n2 + j2) * R2 + b2];
                        T0[(j1 * n2 + j2) * R2 + b2] = s;
                    }
            /* dG3[i3][b2][j3] += sum_{j1,j2} T0[(j1,j2)][b2] dY[(j1,j2)][j3] */
            for (int64_t b2 = 0; b2 < R2; ++b2)
                for (int64_t j3 = 0; j3 < n3; ++j3) {
                    double s = 0.0;
                    for (int64_t q = 0; q < n1 * n2; ++q)
                        s += T0[q * R2 + b2] * dY[q * n3 + j3];
                    gC[b2 * n3 + j3] += s;
                }
            /* dT0[(j1,j2)][b2] = sum_j3 dY[(j1,j2)][j3] C[b2][j3] */
            for (int64_t q = 0; q < n1 * n2; ++q)
                for (int64_t b2 = 0; b2 < R2; ++b2) {
                    double s = 0.0;
                    for (int64_t j3 = 0; j3 < n3; ++j3)
                        s += dY[q * n3 + j3] * (double)C[b2 * n3 + j3];
                    dT0[q * R2 + b2] = s;
                }
            /* dG2[i2][a][j2][b2] += sum_j1 A[j1][a] dT0[(j1,j2)][b2] */
            for (int64_t a = 0; a < R1; ++a)
                for (int64_t j2 = 0; j2 < n2; ++j2)
                    for (int64_t b2 = 0; b2 < R2; ++b2) {
                        double s = 0.0;
                        for (int64_t j1 = 0; j1 < n1; ++j1)
                            s += (double)A[j1 * R1 + a] * dT0[(j1 * n2 + j2) * R2 + b2];
                        gB[(a * n2 + j2) * R2 + b2] += s;
                    }
            /* dG1[i1][j1][a] += sum_{j2,b2} dT0[(j1,j2)][b2] Bm[a][(j2,b2)] */
            for (int64_t j1 = 0; j1 < n1; ++j1)
                for (int64_t a = 0; a < R1; ++a) {
                    double s = 0.0;
                    for (int64_t j2 = 0; j2 < n2; ++j2)
                        for (int64_t b2 = 0; b2 < R2; ++b2)
                            s += dT0[(j1 * n2 + j2) * R2 + b2] * (double)B[(a * n2 + j2) * R2 + b2];
                    gA[j1 * R1 + a] += s;
                }
        }
    }
    free(T0); free(dT0); free(dY); free(map);
    return 0;
}

/* ---- SGD ---------------------------------------------------------------- */

/* Plain SGD, x <- x - lr * g (Section 5: both data sets are trained with SGD;
 * Section 4.2's update of cached rows is read with the same sign and rate). */
void ora_sgd(float *x, const float *g, int64_t count, double lr)
{
    for (int64_t i = 0; i < count; ++i)
        x[i] = (float)((double)x[i] - lr * (double)g[i]);
}

/* ---- dedup -------------------------------------------------------------- */

typedef struct { int64_t key, pos; } kp_t;

static int kp_cmp(const void *pa, const void *pb)
{
    const kp_t *a = (const kp_t *)pa, *b = (const kp_t *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->pos != b->pos) return a->pos < b->pos ? -1 : 1;
    return 0;
}

/* Canonical duplicate-free form of a key stream (the grouping that the "+="
 * of Alg. 2 implies): ascending unique keys, how often each occurs, and the
 * permutation that lists positions grouped by key, positions ascending inside
 * a group.  Keys < 0 are skipped (cached lookups).  Returns the number of
 * unique keys; *n_kept receives the number of positions listed in perm. */
int64_t ora_dedup(const int64_t *keys, int64_t L, int64_t *uniq, int32_t *count,
                  int32_t *perm, int64_t *n_kept)
{
    kp_t *kp = (kp_t *)malloc((size_t)(L > 0 ? L : 1) * sizeof(kp_t));
    int64_t n = 0;
    for (int64_t k = 0; k < L; ++k)
        if (keys[k] >= 0) { kp[n].key = keys[k]; kp[n].pos = k; ++n; }
    qsort(kp, (size_t)n, sizeof(kp_t), kp_cmp);
    int64_t u = 0;
    for (int64_t i = 0; i < n; ++i) {
        perm[i] = (int32_t)kp[i].pos;
        if (i == 0 || kp[i].key != kp[i - 1].key) { uniq[u] = kp[i].key; count[u] = 0; ++u; }
        count[u - 1] += 1;
    }
    *n_kept = n;
    free(kp);
    return u;
}


/* ---- sampled Gaussian initialisation (Section 3.2, Alg. 3) ----------------
 * Every entry of every core is drawn from N(0,1) and redrawn while it lies
 * within two standard deviations of zero (the text wants fewer values close to
 * zero, so the test is on |x|; the listing prints it without the absolute
 * value); then the cores are scaled so that an entry of the reconstructed table
 * has variance 1/(3 num_rows), the N(0, 1/3n) target of Section 3.2: an entry is
 * a sum of R1 R2 products of three core entries of second moment v each, hence
 * scale = (1 / (3 num_rows R1 R2 v^3))^(1/6) with v = E[z^2 | |z| > 2].
 *
 * The random numbers come from a counter-based generator, so that any other
 * implementation can draw the same ones: for core c, element e, attempt t,
 *   h  = mix(mix(seed + GOLD (c + 1)) ^ e),  a = mix(h + T_MUL t),  b = mix(a ^ B_XOR),
 *   u1 = ((a >> 11) + 0.5) 2^-53,  u2 = (b >> 11) 2^-53,
 *   z  = sqrt(-2 ln u1) cos(2 pi u2)            (Box-Muller, in fp64),
 * mix being the finaliser of SplitMix64. */
static uint64_t ora_mix64(uint64_t x)
{
    x ^= x >> 30; x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27; x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}

double ora_sampled_gaussian_draw(uint64_t seed, int core, uint64_t element, int *attempts)
{
    const uint64_t h = ora_mix64(ora_mix64(seed + 0x9E3779B97F4A7C15ull * (uint64_t)(core + 1)) ^ element);
    for (int t = 0;; ++t) {
        const uint64_t a = ora_mix64(h + 0xD1342543DE82EF95ull * (uint64_t)t);
        const uint64_t b = ora_mix64(a ^ 0xA0761D6478BD642Full);
        const double u1 = ((double)(a >> 11) + 0.5) * (1.0 / 9007199254740992.0);
        const double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);
        const double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
        if (fabs(z) > 2.0) {
            if (attempts) *attempts = t + 1;
            return z;
        }
    }
}

double ora_sampled_gaussian_scale(int64_t num_rows, int R1, int R2)
{
    const double phi2 = exp(-2.0) / sqrt(6.283185307179586476925286766559);     /* density of N(0,1) at 2 */
    const double tail = 0.5 * erfc(2.0 / sqrt(2.0));                            /* P(z > 2) */
    const double v = 1.0 + 2.0 * phi2 / tail;                                   /* E[z^2 | |z| > 2] */
    return pow(1.0 / (3.0 * (double)num_rows * (double)R1 * (double)R2 * v * v * v), 1.0 / 6.0);
}

void ora_init_sampled_gaussian(uint64_t seed, int core, int64_t count, double scale, float *out)
{
    for (int64_t e = 0; e < count; ++e)
        out[e] = (float)(ora_sampled_gaussian_draw(seed, core, (uint64_t)e, 0) * scale);
}
