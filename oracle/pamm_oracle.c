/*
 * PAMM oracle: a plain, slow, fp64 CPU statement of what the method computes.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or
 * call this file; it exists so that tests, the smoke check and the benchmark's
 * CPU-baseline leg have something independent to compare the GPU library with.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What it follows (Point-Approximate Matrix Multiplication, Sec. 3.2 and
 * Algorithm 1; the tolerance eps may be infinite, in which case no row is ever
 * dropped and the normalisation factor beta is 1):
 *
 *   Compress(A, k):   I   = k row indices, uniform without replacement   (Alg. 1, Compress, sampling step)
 *                     C_j = A[I_j, :]                                     (Alg. 1, generators)
 *                     alpha(i,j) = <A_i, C_j> / ||C_j||^2                 (Eq. 1)
 *                     f(i) = argmin_j ||A_i - alpha(i,j) C_j||_2
 *                          = argmax_j |csim(A_i, C_j)|                    (Lemma 1)
 *                     alpha_i = alpha(i, f(i))
 *                     e_i = ||A_i - alpha_i C_f(i)||_2 ;  alpha_i <- 0 where
 *                     e_i > eps ||A_i||_2                                 (Eq. 2, neighbourhood condition)
 *                     eta = number of rows dropped, beta = b / (b - eta)  (Sec. 3.2, paragraph on the normalisation factor)
 *   ApproxMM(C, alpha, f, B):
 *                     Btilde_j = sum_{i : f(i) = j} alpha_i B_i           (Sec. 3.2, second stage: the approximate product)
 *                     Otilde   = beta C^T Btilde                          (Alg. 1, ApproxMM; beta as above)
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - Alg. 1 prints argmax(csim) while the definition is argmin residual and
 *     Lemma 1 says argmax |csim|.  The definition wins: the score maximised
 *     here is  s(i,j) = <A_i,C_j>^2 / ||C_j||^2  =  ||A_i||^2 csim^2, which has
 *     the same argmax over j as |csim| because ||A_i|| does not depend on j
 *     (last step of the proof of Lemma 1).  No row norm of A is needed.
 *   - ties: the lowest j wins.
 *   - a zero generator (||C_j|| = 0) scores 0 and yields alpha = 0; a zero row
 *     scores 0 everywhere, so f = 0 and alpha = 0.  No NaN/Inf is produced.
 *   - f is 0-based here (1-based in the paper).
 *   - Alg. 1 prints the neighbourhood test as e > eps; Eq. 2 has e > eps ||A_i||.
 *     Eq. 2 (relative) is taken.  A dropped row keeps its f (Alg. 1 only zeroes
 *     alpha).  If every row is dropped beta is undefined in the paper; 0 here,
 *     so that Otilde = 0.
 *   - the sampler is specified, because the paper fixes only the distribution
 *     (uniform over the k-subsets, no index twice): splitmix64 seeded with `seed`; draw t (t = 0..k-1) takes
 *     r = t + bounded(b - t) where bounded(u) is unbiased rejection sampling
 *     on the 64-bit output (reject x < 2^64 mod u, return x mod u); textbook
 *     Fisher-Yates swap of positions t and r of the identity array; generator
 *     j is the j-th draw (draw order, not sorted).
 *
 * Parity pins (tests/test_oracle_*.py, none of which re-use this code):
 *   sampler      splitmix64 published vectors; permutation at k = b; uniformity chi^2; the bounded
 *                draw, rejection branch included, against exact integer arithmetic on ranges
 *                just above 2^63.  The index stream for a given seed is fixed by the specification
 *                above only: "parity unpinned" by the paper.
 *   f            brute-force argmin of the true residual on tiny inputs (numpy).
 *   alpha        orthogonality of the residual to C_f(i); Pythagoras; alpha = 1 on generators.
 *   Btilde, dW   k = b, C = A gives exactly A^T B; regrouping identity against A~^T B;
 *                k = 1 closed form; error bound of Sec. 3.2.1.
 *   eps, beta    eps = infinity reproduces the unconditioned path; kept rows checked against
 *                Eq. 2 written out in numpy; eps = 0 is uniform column-row sampling
 *                (Sec. 4.1), whose closed form b/k sum_{i in I} A_i^T B_i and whose
 *                unbiasedness over all k-subsets are checked by enumeration; error bound of
 *                Sec. 3.2.1 with dropped rows.
 *
 *   sketch       (the random-projection baseline of Sec. 4.6, at the end of this file; tests/test_oracle_sketch.py)
 *                P = identity gives S = A and exactly A^T B; an orthogonal P gives A^T B; coordinate
 *                selection; the rank-one closed form p p^T A^T B; unbiasedness over Gaussian P.
 *
 * Element types: 0 = IEEE binary32, 1 = bfloat16 (raw 16-bit patterns),
 * 2 = IEEE binary64.  Decoding to double is exact for all three.
 * All matrices are row-major and contiguous.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

/* number of threads the loops below will use (1 without OpenMP) */
int pamm_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void pamm_oracle_set_threads(int t)
{
#ifdef _OPENMP
    if (t > 0) omp_set_num_threads(t);
#else
    (void)t;
#endif
}

static double decode(const void *base, int dtype, size_t idx)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else if (dtype == ORACLE_BF16) {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float v;
        memcpy(&v, &bits, sizeof v);
        return (double)v;
    }
    return ((const double *)base)[idx];
}

/* ---------------------------------------------------------------- sampler */

static uint64_t splitmix64_next(uint64_t *state)
{
    uint64_t z;
    *state += 0x9E3779B97F4A7C15ULL;
    z = *state;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

/* raw generator outputs, exported so that a test can compare them with the published vectors */
void pamm_oracle_splitmix64(uint64_t seed, int64_t count, uint64_t *out)
{
    uint64_t st = seed;
    for (int64_t i = 0; i < count; ++i) out[i] = splitmix64_next(&st);
}

static uint64_t bounded(uint64_t *state, uint64_t u)
{
    /* 2^64 mod u, computed without 128-bit arithmetic */
    uint64_t reject_below = (0ULL - u) % u;
    uint64_t x;
    do {
        x = splitmix64_next(state);
    } while (x < reject_below);
    return x % u;
}

/* `count` consecutive bounded(u) draws from a generator seeded with `seed`, exported so that a test can drive the
   rejection branch (ranges just above 2^63 reject about every second output; the ranges the sampler itself uses,
   below 2^31, reject with probability under 2^-33).  Returns 0, or -1 on bad arguments. */
int pamm_oracle_bounded(uint64_t seed, uint64_t u, int64_t count, uint64_t *out)
{
    if (u == 0 || count < 0 || !out) return -1;
    uint64_t st = seed;
    for (int64_t i = 0; i < count; ++i) out[i] = bounded(&st, u);
    return 0;
}

/* k distinct indices of [0,b), uniform without replacement, in draw order.  Returns 0, or -1 on bad arguments. */
int pamm_oracle_sample(int64_t b, int64_t k, uint64_t seed, int32_t *idx)
{
    if (b < 1 || k < 1 || k > b || !idx) return -1;
    int64_t *a = (int64_t *)malloc((size_t)b * sizeof *a);
    if (!a) return -1;
    for (int64_t i = 0; i < b; ++i) a[i] = i;
    uint64_t st = seed;
    for (int64_t t = 0; t < k; ++t) {
        int64_t r = t + (int64_t)bounded(&st, (uint64_t)(b - t));
        int64_t tmp = a[t];
        a[t] = a[r];
        a[r] = tmp;
        idx[t] = (int32_t)a[t];
    }
    free(a);
    return 0;
}

/* --------------------------------------------------------------- Compress */

/*
 * Inputs : A (b x n, element type dtype), idx[k] (generator rows).
 * Outputs: C      k x n doubles, C_j = A[idx_j]          (Alg. 1, Compress, generator rows)
 *          f      b int32,  0-based assignment            (Lemma 1, lowest j on ties)
 *          alpha  b doubles                               (Eq. 1 at j = f(i))
 *          best   b doubles: s(i, f(i))                   } diagnostics that let a test apply the
 *          second b doubles: max_{j != f(i)} s(i,j)       } "near-tie" exclusion; -1 when k = 1
 *          jsecond b int32: lowest j != f(i) attaining `second`, -1 when k = 1
 *          resid   b doubles: e_i = ||A_i - alpha_i C_f(i)||_2 before the mask       } Eq. 2, both
 *          rownorm b doubles: ||A_i||_2                                               } sides
 *          eta     number of rows dropped by the neighbourhood condition e_i > eps ||A_i||_2
 * eps < 0 stands for eps = infinity (no row dropped).  Any of best/second/jsecond/resid/rownorm/eta may be NULL.
 */
int pamm_oracle_compress(const void *A, int dtype, int64_t b, int64_t n, int64_t k,
                         const int32_t *idx, double eps,
                         double *C, int32_t *f, double *alpha,
                         double *best, double *second, int32_t *jsecond,
                         double *resid, double *rownorm, int64_t *eta)
{
    if (!A || !idx || !C || !f || !alpha || b < 1 || n < 1 || k < 1 || k > b) return -1;
    for (int64_t j = 0; j < k; ++j)
        if (idx[j] < 0 || idx[j] >= b) return -1;

    double *cn2 = (double *)malloc((size_t)k * sizeof *cn2);
    if (!cn2) return -1;
    int64_t dropped = 0;

    for (int64_t j = 0; j < k; ++j) {
        double acc = 0.0;
        for (int64_t l = 0; l < n; ++l) {
            double v = decode(A, dtype, (size_t)idx[j] * (size_t)n + (size_t)l);
            C[j * n + l] = v;
            acc += v * v;
        }
        cn2[j] = acc;                                   /* ||C_j||^2 */
    }

#pragma omp parallel
    {
        double *row = (double *)malloc((size_t)n * sizeof *row);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < b; ++i) {
            for (int64_t l = 0; l < n; ++l) row[l] = decode(A, dtype, (size_t)i * (size_t)n + (size_t)l);

            double s1 = -1.0, d1 = 0.0, s2 = -1.0;
            int64_t j1 = -1, j2 = -1;
            for (int64_t j = 0; j < k; ++j) {
                const double *c = C + j * n;
                double d = 0.0;
                for (int64_t l = 0; l < n; ++l) d += row[l] * c[l];     /* <A_i, C_j> */
                double s = (cn2[j] > 0.0) ? (d * d) / cn2[j] : 0.0;     /* ||A_i||^2 csim^2 */
                if (s > s1) {                   /* strict: lowest j keeps a tie */
                    s2 = s1; j2 = j1;
                    s1 = s;  j1 = j;  d1 = d;
                } else if (s > s2) {
                    s2 = s;  j2 = j;
                }
            }
            f[i] = (int32_t)j1;
            double a = (cn2[j1] > 0.0) ? d1 / cn2[j1] : 0.0;           /* Eq. 1 */
            if (best) best[i] = s1;
            if (second) second[i] = s2;
            if (jsecond) jsecond[i] = (int32_t)j2;

            /* Eq. 2: the residual of the representative, formed as the vector it is */
            const double *c = C + j1 * n;
            double e2 = 0.0, a2 = 0.0;
            for (int64_t l = 0; l < n; ++l) {
                double r = row[l] - a * c[l];
                e2 += r * r;
                a2 += row[l] * row[l];
            }
            double e = sqrt(e2), na = sqrt(a2);
            if (resid) resid[i] = e;
            if (rownorm) rownorm[i] = na;
            if (eps >= 0.0 && e > eps * na) {                          /* neighbourhood condition fails: drop the row */
                a = 0.0;
#pragma omp atomic
                dropped += 1;
            }
            alpha[i] = a;
        }
        free(row);
    }
    free(cn2);
    if (eta) *eta = dropped;
    return 0;
}

/* beta = b / (b - eta) (Sec. 3.2); 0 when every row was dropped */
double pamm_oracle_beta(int64_t b, int64_t eta)
{
    return (eta < b) ? (double)b / (double)(b - eta) : 0.0;
}

/* --------------------------------------------------------------- ApproxMM */

/*
 * Inputs : C (k x n doubles), f (b), alpha (b doubles), B (b x m, element type dtype).
 * Outputs: Btilde k x m doubles, Btilde_j = sum_{i: f(i)=j} alpha_i B_i, rows added in increasing i;
 *          O      n x m doubles, O = beta C^T Btilde, plain triple loop with j innermost-in-order
 *                 (beta = 1 when no row was dropped).
 */
int pamm_oracle_grad(const double *C, const int32_t *f, const double *alpha,
                     const void *B, int dtype,
                     int64_t b, int64_t n, int64_t k, int64_t m, double beta,
                     double *Btilde, double *O)
{
    if (!C || !f || !alpha || !B || !Btilde || !O || b < 1 || n < 1 || k < 1 || m < 1) return -1;
    for (int64_t i = 0; i < b; ++i)
        if (f[i] < 0 || f[i] >= k) return -1;

    memset(Btilde, 0, (size_t)k * (size_t)m * sizeof *Btilde);

    /* every thread owns a range of columns and walks the rows in order, so each
       element of Btilde is accumulated in increasing i whatever the thread count */
#pragma omp parallel
    {
#ifdef _OPENMP
        int nt = omp_get_num_threads(), me = omp_get_thread_num();
#else
        int nt = 1, me = 0;
#endif
        int64_t c0 = (m * me) / nt, c1 = (m * (me + 1)) / nt;
        for (int64_t i = 0; i < b; ++i) {
            double a = alpha[i];
            double *dst = Btilde + (int64_t)f[i] * m;
            for (int64_t c = c0; c < c1; ++c)
                dst[c] += a * decode(B, dtype, (size_t)i * (size_t)m + (size_t)c);
        }
    }

#pragma omp parallel for schedule(static)
    for (int64_t l = 0; l < n; ++l) {
        double *out = O + l * m;
        for (int64_t c = 0; c < m; ++c) out[c] = 0.0;
        for (int64_t j = 0; j < k; ++j) {
            double cjl = C[j * n + l];
            const double *bt = Btilde + j * m;
            for (int64_t c = 0; c < m; ++c) out[c] += cjl * bt[c];
        }
        for (int64_t c = 0; c < m; ++c) out[c] *= beta;
    }
    return 0;
}

/* ------------------------------------------------ comparison: low-rank sketch */

/*
 * The random-projection baseline of the ablation (Sec. 4.6): instead of (C, f, alpha) the layer keeps the
 * sketch S = A P of its input, P an n x r random matrix with E[P P^T] = I, and the weight gradient is
 * estimated as P (S^T B) = (P P^T) A^T B.  The random numbers are an input: P is passed through its
 * transpose Pt (r x n, row-major), so that row j of Pt is the j-th sketch direction.
 *
 * pamm_oracle_sketch:       S[i][j] = <A_i, Pt_j>                       (b x r doubles, not rounded)
 * pamm_oracle_sketch_grad:  G = S^T B  (r x m),  O = Pt^T G  (n x m),   rows added in increasing i / j.
 * The stored sketch has an element type of its own (sdtype): the caller rounds S to what the layer keeps.
 */
int pamm_oracle_sketch(const void *A, int dtype, const void *Pt, int pdtype,
                       int64_t b, int64_t n, int64_t r, double *S)
{
    if (!A || !Pt || !S || b < 1 || n < 1 || r < 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < b; ++i)
        for (int64_t j = 0; j < r; ++j) {
            double d = 0.0;
            for (int64_t l = 0; l < n; ++l)
                d += decode(A, dtype, (size_t)i * (size_t)n + (size_t)l) * decode(Pt, pdtype, (size_t)j * (size_t)n + (size_t)l);
            S[i * r + j] = d;
        }
    return 0;
}

int pamm_oracle_sketch_grad(const void *Pt, int pdtype, const void *S, int sdtype,
                            const void *B, int dtype,
                            int64_t b, int64_t n, int64_t r, int64_t m,
                            double *G, double *O)
{
    if (!Pt || !S || !B || !G || !O || b < 1 || n < 1 || r < 1 || m < 1) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < r; ++j) {
        double *g = G + j * m;
        for (int64_t c = 0; c < m; ++c) g[c] = 0.0;
        for (int64_t i = 0; i < b; ++i) {
            double s = decode(S, sdtype, (size_t)i * (size_t)r + (size_t)j);
            for (int64_t c = 0; c < m; ++c) g[c] += s * decode(B, dtype, (size_t)i * (size_t)m + (size_t)c);
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t l = 0; l < n; ++l) {
        double *out = O + l * m;
        for (int64_t c = 0; c < m; ++c) out[c] = 0.0;
        for (int64_t j = 0; j < r; ++j) {
            double p = decode(Pt, pdtype, (size_t)j * (size_t)n + (size_t)l);     /* P[l][j] */
            const double *g = G + j * m;
            for (int64_t c = 0; c < m; ++c) out[c] += p * g[c];
        }
    }
    return 0;
}
