/*
 * ZipML CPU oracle -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, scalar implementation of double-sampled low-precision
 * minibatch SGD for least squares, written from the paper
 * ("ZipML: Training Models with End-to-End Low Precision", arXiv 1611.05402).
 * It exists so that the GPU library can be checked against something that can
 * be read next to the paper.  It shares no source, header, table or helper
 * with the HIP library and nothing in the product path may call it: only the
 * tests, the smoke check and the benchmark's cpu_baseline leg do.
 *
 * Conventions
 *   - "levels" is a per-feature table L[j][c], c = 0..K-1, K = 2^bits,
 *     non-decreasing in c (Sec. 2.1: separators of the normalised range;
 *     Supp. A.3 "Column Scaling": one range per feature shared by all rows).
 *   - codes are canonical row-major uint8 [n][d].
 *   - A is row-major fp32 with leading dimension lda.
 *   - Every floating-point operation that decides an integer (a quantised
 *     code) is written as single IEEE fp32/fp64 operations in a fixed order;
 *     build with -ffp-contract=off so the compiler cannot fuse them.
 *   - Everything else is evaluated in fp64.
 *
 * Pins (see tests/, "-m 'not gpu'"): Philox known answers; exact two-outcome
 * expectation and variance (b-x)(x-a); the paper's 0.7 -> {0,1} example;
 * naive-estimator bias = diag(err) x and double-sampled bias = 0 by full
 * enumeration; on-grid data == textbook minibatch SGD; convergence to the
 * normal-equations solution; DP == brute force over all level subsets; the
 * l2 term == textbook ridge SGD and its closed form; the proximal step ==
 * brute-force minimisation of its definition and the lasso / ridge / box
 * closed forms of an orthogonal design; the greedy intervals == a partition
 * worked out by hand, within twice the optimum of the dynamic program, and
 * == the optimum on clustered data; one end-to-end step at minibatches of 96
 * to 200 samples == an independent fp64 step (integer dots, residual bits,
 * the mean gradient to one unit in the last place, Q4 and the update from
 * that gradient); the all-cores epoch == the plain epoch.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------- */
/* Counter-based random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw,  */
/* "Parallel random numbers: as easy as 1, 2, 3", SC'11).  The paper is      */
/* silent on the generator; a counter-based one makes each stochastic        */
/* decision a pure function of (seed, epoch, row, col, stream).              */
/* ------------------------------------------------------------------------- */
void zo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Stream ids: 1, 2 = the two independent sample quantisations Q1, Q2
 * (Sec. 2.2, eq. (5)); 3 = model quantisation Q3; 4 = gradient quantisation
 * Q4 (Supp. E).  For streams 1, 2 "row" is the sample index; for 3, 4 it is
 * the step index inside the epoch.
 * Key = seed (low, high word).  Counter = (row low, row high, col / 4,
 * epoch * 256 + stream); the output word col % 4 belongs to that column.
 * The uniform is the top 24 bits scaled to [0, 1): exact in fp32. */
float zo_uniform24(uint64_t seed, uint32_t epoch, uint64_t row, uint32_t col, uint32_t stream)
{
    uint32_t ctr[4], key[2], out[4];
    key[0] = (uint32_t)seed;
    key[1] = (uint32_t)(seed >> 32);
    ctr[0] = (uint32_t)row;
    ctr[1] = (uint32_t)(row >> 32);
    ctr[2] = col >> 2;
    ctr[3] = (epoch << 8) | stream;
    zo_philox4x32_10(ctr, key, out);
    return (float)(out[col & 3u] >> 8) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------------- */
/* Column scaling (Supp. A.3 "Column Scaling"): per-feature min and max over */
/* all samples.  symmetric != 0 gives the paper's M_j = max(|min|, |max|),   */
/* i.e. the range [-M_j, M_j]; otherwise the range is [min_j, max_j]         */
/* (Sec. 3 works on a min-max normalised [0,1]).                             */
/* ------------------------------------------------------------------------- */
void zo_col_range(const float *A, int64_t n, int64_t d, int64_t lda, int symmetric,
                  float *lo, float *hi)
{
    for (int64_t j = 0; j < d; ++j) {
        float mn = A[j], mx = A[j];
        for (int64_t i = 1; i < n; ++i) {
            float v = A[i * lda + j];
            if (v < mn) mn = v;
            if (v > mx) mx = v;
        }
        if (symmetric) {
            float m = fabsf(mn) > fabsf(mx) ? fabsf(mn) : fabsf(mx);
            mn = -m;
            mx = m;
        }
        lo[j] = mn;
        hi[j] = mx;
    }
}

/* Uniform levels (Sec. 2.1): K = 2^bits evenly spaced points on [lo_j, hi_j],
 * evaluated in fp64 and rounded once.  c = K-1 gives hi_j exactly. */
void zo_levels_uniform(const float *lo, const float *hi, int64_t d, int bits, float *levels)
{
    int K = 1 << bits;
    for (int64_t j = 0; j < d; ++j) {
        double l = (double)lo[j], w = (double)hi[j] - (double)lo[j];
        for (int c = 0; c < K; ++c)
            levels[j * K + c] = (float)(l + ((double)c * w) / (double)(K - 1));
    }
}

/* ------------------------------------------------------------------------- */
/* Variance-optimal levels (Sec. 3).                                         */
/* ------------------------------------------------------------------------- */

/* One scan of the data (Sec. 3.2 "Discretization"): normalise each value of
 * column j to t = (a - lo_j)/(hi_j - lo_j) in [0,1], drop it in one of M
 * equal bins [m/M, (m+1)/M) (the last one closed) and accumulate per bin the
 * count, sum of t and sum of t^2.  hist is [d][M][3] doubles.  A column with
 * hi_j == lo_j puts everything in bin 0 with t = 0. */
void zo_hist_moments(const float *A, int64_t n, int64_t d, int64_t lda,
                     const float *lo, const float *hi, int M, double *hist)
{
    memset(hist, 0, sizeof(double) * (size_t)d * (size_t)M * 3);
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < d; ++j) {
            double w = (double)hi[j] - (double)lo[j];
            double t = 0.0;
            if (w > 0.0) {
                t = ((double)A[i * lda + j] - (double)lo[j]) / w;
                if (t < 0.0) t = 0.0;
                if (t > 1.0) t = 1.0;
            }
            int m = (int)(t * (double)M);
            if (m > M - 1) m = M - 1;
            double *h = hist + ((size_t)j * M + m) * 3;
            h[0] += 1.0;
            h[1] += t;
            h[2] += t * t;
        }
    }
}

/* Per-bin moments for arbitrary sorted candidate endpoints cand[0..M]
 * (cand[0] = 0, cand[M] = 1), bins [cand_m, cand_{m+1}), last one closed.
 * Used for the exact algorithm where the candidates are the data points
 * themselves (Lemma 3 / Sec. 3.1). */
void zo_bin_moments(const double *t, int64_t N, const double *cand, int M, double *mom /*[M][3]*/)
{
    memset(mom, 0, sizeof(double) * (size_t)M * 3);
    for (int64_t i = 0; i < N; ++i) {
        int m = 0;
        while (m + 1 < M && t[i] >= cand[m + 1]) ++m;
        mom[m * 3 + 0] += 1.0;
        mom[m * 3 + 1] += t[i];
        mom[m * 3 + 2] += t[i] * t[i];
    }
}

/* Dynamic program of Sec. 3.1 restricted to candidate endpoints (Sec. 3.2
 * "Dynamic Programming with Candidate Points").
 *   V(j, m) = sum over points t in [cand_j, cand_m) of (cand_m - t)(t - cand_j)
 *   T(1, m) = V(0, m);  T(k, m) = min_{k-1 <= j <= m-1} T(k-1, j) + V(j, m)
 * where k counts intervals.  Returns T(s, M) (the total, not the mean,
 * variance) and writes the s+1 chosen endpoint indices 0 = idx[0] < ... <
 * idx[s] = M.  Ties go to the smallest j.  Needs M >= s >= 1. */
double zo_dp_levels(const double *mom /*[M][3]*/, const double *cand /*[M+1]*/, int M, int s,
                    int *idx /*[s+1]*/)
{
    double *C = calloc((size_t)M + 1, sizeof(double));
    double *S1 = calloc((size_t)M + 1, sizeof(double));
    double *S2 = calloc((size_t)M + 1, sizeof(double));
    for (int m = 0; m < M; ++m) {
        C[m + 1] = C[m] + mom[m * 3 + 0];
        S1[m + 1] = S1[m] + mom[m * 3 + 1];
        S2[m + 1] = S2[m] + mom[m * 3 + 2];
    }
    size_t W = (size_t)M + 1;
    double *T = malloc(sizeof(double) * W * ((size_t)s + 1));
    int *arg = malloc(sizeof(int) * W * ((size_t)s + 1));
    for (size_t q = 0; q < W * ((size_t)s + 1); ++q) { T[q] = INFINITY; arg[q] = -1; }
#define ZO_V(j, m) (-(S2[m] - S2[j]) + (cand[j] + cand[m]) * (S1[m] - S1[j]) \
                    - cand[j] * cand[m] * (C[m] - C[j]))
    for (int m = 1; m <= M; ++m) { T[1 * W + m] = ZO_V(0, m); arg[1 * W + m] = 0; }
    for (int k = 2; k <= s; ++k) {
        for (int m = k; m <= M; ++m) {
            double best = INFINITY;
            int bj = -1;
            for (int j = k - 1; j <= m - 1; ++j) {
                double v = T[(size_t)(k - 1) * W + j] + ZO_V(j, m);
                if (v < best) { best = v; bj = j; }
            }
            T[(size_t)k * W + m] = best;
            arg[(size_t)k * W + m] = bj;
        }
    }
#undef ZO_V
    double total = T[(size_t)s * W + M];
    int m = M;
    for (int k = s; k >= 1; --k) {
        idx[k] = m;
        m = arg[(size_t)k * W + m];
    }
    idx[0] = 0;
    free(C); free(S1); free(S2); free(T); free(arg);
    return total;
}

/* Per-feature variance-optimal level sets from the M-bin moments: s = K-1
 * intervals on the grid m/M, L[j][c] = lo_j + (hi_j - lo_j) * G[j][c] / M.
 * mean_variance (may be NULL) receives the objective MV of eq. (6) averaged
 * over all features, in normalised units. */
void zo_levels_optimal(const double *hist, const float *lo, const float *hi, int64_t d, int bits,
                       int M, float *levels, uint16_t *grid_idx, double *mean_variance)
{
    int K = 1 << bits, s = K - 1;
    double *cand = malloc(sizeof(double) * ((size_t)M + 1));
    int *idx = malloc(sizeof(int) * ((size_t)s + 1));
    for (int m = 0; m <= M; ++m) cand[m] = (double)m / (double)M;
    double mv = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        const double *mom = hist + (size_t)j * M * 3;
        double cnt = 0.0;
        for (int m = 0; m < M; ++m) cnt += mom[m * 3];
        double total = zo_dp_levels(mom, cand, M, s, idx);
        if (cnt > 0.0) mv += total / cnt;
        double l = (double)lo[j], w = (double)hi[j] - (double)lo[j];
        for (int c = 0; c < K; ++c) {
            if (grid_idx) grid_idx[j * K + c] = (uint16_t)idx[c];
            levels[j * K + c] = (float)(l + (w * (double)idx[c]) / (double)M);
        }
    }
    if (mean_variance) *mean_variance = mv / (double)d;
    free(cand);
    free(idx);
}

/* Greedy merging of intervals (supplement, "A Greedy Algorithm for Finding
 * Quantization Points", Algorithm 1), run on the M bins of the candidate
 * grid instead of on single points: the starting partition has one interval
 * per bin, an interval carries the moments (count, sum t, sum t^2) of its
 * points, and the error of an interval [a, b] is
 *     err = sum over its points of (b - t)(t - a) = -S2 + (a + b) S1 - a b S0.
 * While more than 2 (1 + gamma) k + delta intervals are left: consecutive
 * intervals are paired up (an odd one at the end stays as it is), every pair
 * gets the error of the merged interval (moments of the left one plus those
 * of the right one), the q = (1 + gamma) k pairs with the largest error stay
 * split (equal errors: the pair further left first), all others are merged.
 * gamma = 1, delta = 1 here: at most 4 k + 1 intervals come out (with
 * delta = 0 a partition of 4 k + 1 intervals would never shrink), and their
 * error is at most 2 OPT_k (the supplement's theorem).
 * edge[0..P] receives the bin-edge indices of the partition (0 and M among
 * them), mom[P][3] its moments; returns P. */
int zo_greedy_intervals(const double *hist /*[M][3]*/, int M, int k, int *edge /*[M+1]*/,
                        double *mom /*[M][3]*/)
{
    const int q = 2 * k, limit = 4 * k + 1;
    int P = M;
    for (int m = 0; m <= M; ++m) edge[m] = m;
    memcpy(mom, hist, sizeof(double) * (size_t)M * 3);
    double *e = malloc(sizeof(double) * (size_t)(M / 2 + 1));
    int *keep = malloc(sizeof(int) * (size_t)(M / 2 + 1));
    while (P > limit) {
        const int pairs = P / 2;
        for (int i = 0; i < pairs; ++i) {
            const double a = (double)edge[2 * i] / (double)M, b = (double)edge[2 * i + 2] / (double)M;
            const double s0 = mom[(2 * i) * 3 + 0] + mom[(2 * i + 1) * 3 + 0];
            const double s1 = mom[(2 * i) * 3 + 1] + mom[(2 * i + 1) * 3 + 1];
            const double s2 = mom[(2 * i) * 3 + 2] + mom[(2 * i + 1) * 3 + 2];
            e[i] = -s2 + (a + b) * s1 - a * b * s0;
        }
        /* the q pairs with the largest error: pair i stays split if fewer than q pairs come before it
         * in the order "larger error first, then further left" */
        for (int i = 0; i < pairs; ++i) {
            int before = 0;
            for (int j = 0; j < pairs; ++j)
                if (e[j] > e[i] || (e[j] == e[i] && j < i)) ++before;
            keep[i] = before < q;
        }
        int out = 0;
        for (int i = 0; i < pairs; ++i) {
            if (keep[i]) {
                for (int h = 0; h < 2; ++h) {
                    edge[out] = edge[2 * i + h];
                    for (int c = 0; c < 3; ++c) mom[out * 3 + c] = mom[(2 * i + h) * 3 + c];
                    ++out;
                }
            } else {
                const double s0 = mom[(2 * i) * 3 + 0] + mom[(2 * i + 1) * 3 + 0];
                const double s1 = mom[(2 * i) * 3 + 1] + mom[(2 * i + 1) * 3 + 1];
                const double s2 = mom[(2 * i) * 3 + 2] + mom[(2 * i + 1) * 3 + 2];
                edge[out] = edge[2 * i];
                mom[out * 3 + 0] = s0; mom[out * 3 + 1] = s1; mom[out * 3 + 2] = s2;
                ++out;
            }
        }
        if (P & 1) {
            edge[out] = edge[P - 1];
            for (int c = 0; c < 3; ++c) mom[out * 3 + c] = mom[(P - 1) * 3 + c];
            ++out;
        }
        edge[out] = M;
        P = out;
    }
    free(e);
    free(keep);
    return P;
}

/* Levels from the greedy intervals: their end points are the candidates of
 * the dynamic program (Sec. 3.2, "2-Approximation in Almost-Linear Time").
 * Same outputs as zo_levels_optimal; grid indices refer to the M-bin grid. */
void zo_levels_greedy(const double *hist, const float *lo, const float *hi, int64_t d, int bits,
                      int M, float *levels, uint16_t *grid_idx, double *mean_variance)
{
    int K = 1 << bits, s = K - 1;
    int *edge = malloc(sizeof(int) * ((size_t)M + 1));
    double *mom = malloc(sizeof(double) * (size_t)M * 3);
    double *cand = malloc(sizeof(double) * ((size_t)M + 1));
    int *idx = malloc(sizeof(int) * ((size_t)s + 1));
    double mv = 0.0;
    for (int64_t j = 0; j < d; ++j) {
        const double *h = hist + (size_t)j * M * 3;
        double cnt = 0.0;
        for (int m = 0; m < M; ++m) cnt += h[m * 3];
        const int P = zo_greedy_intervals(h, M, s, edge, mom);
        for (int m = 0; m <= P; ++m) cand[m] = (double)edge[m] / (double)M;
        double total = zo_dp_levels(mom, cand, P, s, idx);
        if (cnt > 0.0) mv += total / cnt;
        double l = (double)lo[j], w = (double)hi[j] - (double)lo[j];
        for (int c = 0; c < K; ++c) {
            const int g = edge[idx[c]];
            if (grid_idx) grid_idx[j * K + c] = (uint16_t)g;
            levels[j * K + c] = (float)(l + (w * (double)g) / (double)M);
        }
    }
    if (mean_variance) *mean_variance = mv / (double)d;
    free(edge); free(mom); free(cand); free(idx);
}

/* ------------------------------------------------------------------------- */
/* Stochastic quantisation of samples (Sec. 2.1; Supp. A.3).                 */
/* ------------------------------------------------------------------------- */

/* Bracket v by two neighbouring levels and return the lower index l and the
 * probability frac of rounding up.  Three fp32 operations decide frac. */
static int bracket(const float *L, int K, float v, float *frac)
{
    if (v < L[0]) v = L[0];
    if (v > L[K - 1]) v = L[K - 1];
    int l = 0;
    for (int c = 1; c <= K - 2 && L[c] <= v; ++c) l = c; /* levels are non-decreasing */
    float w = L[l + 1] - L[l];
    float num = v - L[l];
    *frac = (w > 0.0f) ? num / w : 0.0f;
    return l;
}

/* Two independent quantisations of every sample (Sec. 2.2): copy k uses
 * stream k.  code = l + [u < frac], so E[L[code]] = v. */
void zo_quantize(const float *A, int64_t n, int64_t d, int64_t lda, int64_t row0,
                 const float *levels, int bits, uint64_t seed, uint32_t epoch,
                 uint8_t *codes1, uint8_t *codes2)
{
    int K = 1 << bits;
    for (int64_t i = 0; i < n; ++i) {
        for (int64_t j = 0; j < d; ++j) {
            float frac;
            int l = bracket(levels + j * K, K, A[i * lda + j], &frac);
            float u1 = zo_uniform24(seed, epoch, (uint64_t)(row0 + i), (uint32_t)j, 1);
            float u2 = zo_uniform24(seed, epoch, (uint64_t)(row0 + i), (uint32_t)j, 2);
            codes1[i * d + j] = (uint8_t)(l + (u1 < frac ? 1 : 0));
            codes2[i * d + j] = (uint8_t)(l + (u2 < frac ? 1 : 0));
        }
    }
}

/* The lower level index and the round-up probability of one value: lets a
 * test enumerate the two outcomes exactly. */
int zo_bracket(const float *L, int bits, float v, float *frac)
{
    return bracket(L, 1 << bits, v, frac);
}

/* ------------------------------------------------------------------------- */
/* Row-scaled sign-magnitude quantiser for model and gradient vectors        */
/* (Supp. A.3 eq. (quant2) with "Row Scaling" M = ||v||_2).  s intervals on  */
/* [0,1] for the magnitude; s = 2^(bits-1) - 1 so that the signed code fits  */
/* in `bits` bits.                                                           */
/* ------------------------------------------------------------------------- */

/* ||v||_2 as fp32: squares are exact in fp64; they are summed in fp64 in a
 * fixed adjacent-pair tree over the power-of-two padded vector, so that any
 * implementation following the same tree gets the same bits. */
float zo_norm2(const float *v, int64_t d)
{
    int64_t P = 1;
    while (P < d) P <<= 1;
    double *a = calloc((size_t)P, sizeof(double));
    for (int64_t j = 0; j < d; ++j) a[j] = (double)v[j] * (double)v[j];
    for (int64_t stride = 1; stride < P; stride <<= 1)
        for (int64_t i = 0; i + stride < P; i += 2 * stride)
            a[i] = a[i] + a[i + stride];
    double S = a[0];
    free(a);
    return (float)sqrt(S);
}

/* Signed integer code m in [-s, s] with E[M * m / s] = v.  u is the uniform
 * for this element. */
static int32_t qvec_code(float v, float M, int s, float u)
{
    if (!(M > 0.0f)) return 0;
    float a = fabsf(v);
    float t = a / M;
    float y = t * (float)s;
    int l = (int)floorf(y);
    if (l > s - 1) l = s - 1;
    float frac = y - (float)l;
    int mag = l + (u < frac ? 1 : 0);
    return v < 0.0f ? -mag : mag;
}

/* Q(v, s) of a whole vector: codes[j] in [-s, s]; returns the scale
 * sigma = M / s so that Q(v)_j = sigma * codes[j].  stream = 3 (model) or
 * 4 (gradient); step keys the draw. */
float zo_quantize_vec(const float *v, int64_t d, int bits, uint64_t seed, uint32_t epoch,
                      uint64_t step, uint32_t stream, int32_t *codes)
{
    int s = (1 << (bits - 1)) - 1;
    float M = zo_norm2(v, d);
    for (int64_t j = 0; j < d; ++j) {
        float u = zo_uniform24(seed, epoch, step, (uint32_t)j, stream);
        codes[j] = qvec_code(v[j], M, s, u);
    }
    return (M > 0.0f) ? M / (float)s : 0.0f;
}

/* Same with the uniforms supplied by the caller (for exact enumeration). */
float zo_quantize_vec_u(const float *v, int64_t d, int bits, const float *u, int32_t *codes)
{
    int s = (1 << (bits - 1)) - 1;
    float M = zo_norm2(v, d);
    for (int64_t j = 0; j < d; ++j) codes[j] = qvec_code(v[j], M, s, u[j]);
    return (M > 0.0f) ? M / (float)s : 0.0f;
}

/* ------------------------------------------------------------------------- */
/* Gradient estimators for one sample (Sec. 2.2), in fp64.                   */
/* ------------------------------------------------------------------------- */

/* Naive single-quantisation estimator  Q(a) Q(a)^T x - Q(a) b. */
void zo_grad_naive(const uint8_t *code, const float *levels, int64_t d, int bits,
                   const double *x, double b, double *g)
{
    int K = 1 << bits;
    double z = 0.0;
    for (int64_t j = 0; j < d; ++j) z += (double)levels[j * K + code[j]] * x[j];
    for (int64_t j = 0; j < d; ++j) g[j] = (double)levels[j * K + code[j]] * (z - b);
}

/* Double-sampled estimator of eq. (5):  Q1(a) (Q2(a)^T x - b). */
void zo_grad_double(const uint8_t *code1, const uint8_t *code2, const float *levels, int64_t d,
                    int bits, const double *x, double b, double *g)
{
    int K = 1 << bits;
    double z = 0.0;
    for (int64_t j = 0; j < d; ++j) z += (double)levels[j * K + code2[j]] * x[j];
    for (int64_t j = 0; j < d; ++j) g[j] = (double)levels[j * K + code1[j]] * (z - b);
}

/* ------------------------------------------------------------------------- */
/* One epoch of double-sampled minibatch SGD on F(x) = 1/(2n) sum_i          */
/* (a_i^T x - b_i)^2  (Sec. 2, eq. (5); minibatch = mean over the batch;     */
/* sequential contiguous batches).  x is the fp32 master model, in/out.      */
/*                                                                           */
/* symmetric != 0 uses the averaged estimator of the footnote in Supp. B.2:  */
/*   1/2 [ Q1 (Q2^T x - b) + Q2 (Q1^T x - b) ].                              */
/*                                                                           */
/* Full-precision-model mode (this function): every operation inside a step  */
/* is fp64; the model is rounded to fp32 once per step, at the update.       */
/* With l2 = c the objective has the extra term (c/2)||x||^2 of the least-   */
/* squares SVM (labels +-1) and a step is  x <- x - lr (g + c x).            */
/* ------------------------------------------------------------------------- */
/* Proximal operator of gamma * R at v (Sec. 2, the update x <- prox_{gamma R}(x - gamma g)):
 * argmin_u 1/2 (u - v)^2 + gamma R(u), coordinate by coordinate, for the separable regularisers
 *   kind 1: R(x) = coef * ||x||_1            -> soft threshold at gamma * coef
 *   kind 2: R(x) = coef / 2 * ||x||_2^2      -> v / (1 + gamma * coef)
 *   kind 3: R = indicator of ||x||_inf <= coef (a constraint) -> clamp to [-coef, coef]
 *   kind 0: R = 0. */
double zo_prox(double v, int kind, double gamma, double coef)
{
    if (kind == 1) {
        double t = gamma * coef;
        return v > t ? v - t : v < -t ? v + t : 0.0;
    }
    if (kind == 2) return v / (1.0 + gamma * coef);
    if (kind == 3) return v > coef ? coef : v < -coef ? -coef : v;
    return v;
}

void zo_sgd_epoch(const uint8_t *codes1, const uint8_t *codes2, const float *levels,
                  const float *b, int64_t n, int64_t d, int bits, float *x, int64_t batch,
                  float lr, int symmetric, float l2, int prox, float prox_coef)
{
    int K = 1 << bits;
    double *r2 = malloc(sizeof(double) * (size_t)batch); /* residuals from copy 2 */
    double *r1 = malloc(sizeof(double) * (size_t)batch); /* residuals from copy 1 */
    double *g = malloc(sizeof(double) * (size_t)d);
    for (int64_t t = 0; t < n / batch; ++t) {
        const uint8_t *c1 = codes1 + t * batch * d, *c2 = codes2 + t * batch * d;
        const float *bb = b + t * batch;
        for (int64_t i = 0; i < batch; ++i) {
            double z2 = 0.0, z1 = 0.0;
            for (int64_t j = 0; j < d; ++j) {
                z2 += (double)levels[j * K + c2[i * d + j]] * (double)x[j];
                z1 += (double)levels[j * K + c1[i * d + j]] * (double)x[j];
            }
            r2[i] = z2 - (double)bb[i];
            r1[i] = z1 - (double)bb[i];
        }
        for (int64_t j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int64_t i = 0; i < batch; ++i) {
                if (symmetric)
                    acc += 0.5 * ((double)levels[j * K + c1[i * d + j]] * r2[i] +
                                  (double)levels[j * K + c2[i * d + j]] * r1[i]);
                else
                    acc += (double)levels[j * K + c1[i * d + j]] * r2[i];
            }
            g[j] = acc / (double)batch;
        }
        /* l2 = c > 0: least-squares SVM, the gradient gets the additional term c x
         * ("Extension to Classification Models"). */
        for (int64_t j = 0; j < d; ++j) {
            double v = (double)x[j] - (double)lr * (g[j] + (double)l2 * (double)x[j]);
            x[j] = (float)zo_prox(v, prox, (double)lr, (double)prox_coef);
        }
    }
    free(r2); free(r1); free(g);
}

/* The same epoch (eq. (5), plain estimator, no regulariser) with the rows of each minibatch
 * shared out over `threads` host threads: thread k takes the k-th contiguous share of the rows,
 * forms their residuals and its own partial sum of the gradient in fp64; the partial sums are
 * added in thread order.  With one thread it is zo_sgd_epoch operation for operation; with more
 * only the association of the fp64 sum over the batch changes.  Returns the number of threads the
 * parallel regions ran with. */
int zo_sgd_epoch_threads(const uint8_t *codes1, const uint8_t *codes2, const float *levels,
                         const float *b, int64_t n, int64_t d, int bits, float *x, int64_t batch,
                         float lr, int threads)
{
    int K = 1 << bits;
    if (threads < 1) threads = 1;
    double *gp = malloc(sizeof(double) * (size_t)d * (size_t)threads);
    int used = 1;
    for (int64_t t = 0; t < n / batch; ++t) {
        const uint8_t *c1 = codes1 + t * batch * d, *c2 = codes2 + t * batch * d;
        const float *bb = b + t * batch;
#pragma omp parallel num_threads(threads)
        {
            int k = 0, nt = 1;
#ifdef _OPENMP
            k = omp_get_thread_num();
            nt = omp_get_num_threads();
#endif
            if (k == 0) used = nt;
            int64_t i0 = batch * k / nt, i1 = batch * (k + 1) / nt;
            double *g = gp + (size_t)k * (size_t)d;
            for (int64_t j = 0; j < d; ++j) g[j] = 0.0;
            for (int64_t i = i0; i < i1; ++i) {
                double z = 0.0;
                for (int64_t j = 0; j < d; ++j)
                    z += (double)levels[j * K + c2[i * d + j]] * (double)x[j];
                double r = z - (double)bb[i];
                for (int64_t j = 0; j < d; ++j) g[j] += (double)levels[j * K + c1[i * d + j]] * r;
            }
        }
        for (int64_t j = 0; j < d; ++j) {
            double acc = 0.0;
            for (int k = 0; k < used; ++k) acc += gp[(size_t)k * (size_t)d + j];
            x[j] = (float)((double)x[j] - (double)lr * (acc / (double)batch));
        }
    }
    free(gp);
    return used;
}

/* ------------------------------------------------------------------------- */
/* End-to-end low precision (Supp. C-E):                                     */
/*   g = Q4( Q1(a) ( Q2(a)^T Q3(x) - b ) ),  x <- x - lr g  in full          */
/* precision.  model_bits > 0 switches Q3 on, grad_bits > 0 switches Q4 on   */
/* (model_bits must be > 0 here).  Discrete decisions depend on floating-    */
/* point intermediates, so every operation below is a stated fp32/fp64 op in */
/* a stated order:                                                           */
/*   - sample values in the dot product are  grid_lo + grid_step * G[j][c]   */
/*     with integer grid indices G (the same lo and step for all features),  */
/*     so the dot is an exact integer sum  acc_i = sum_j G[j][c2_ij] * m_j;  */
/*   - z_i = fp32( sigma * (lo * sum_j m_j + step * acc_i) ) in fp64;        */
/*   - r_i = z_i - b_i in fp32;                                              */
/*   - g_j = (1/B) sum_i L[j][c1_ij] r_i, the mean of eq. (5), rounded to   */
/*     fp32 once: every product of two fp32 numbers is exact in fp64, the    */
/*     sum runs in fp64 in sample order and is divided by the batch size in  */
/*     fp64 (the paper fixes no order; fp64 makes the order immaterial to    */
/*     the fp32 result except in a 2^-29 fraction of the cases);             */
/*   - Q4 and the update in fp32, multiply then subtract.                    */
/* Optional debug outputs (any may be NULL) capture the LAST step:           */
/*   dbg_m[d] model codes, dbg_acc[batch] integer dots, dbg_r[batch],        */
/*   dbg_g[d] gradient before Q4, dbg_gq[d] gradient codes.                  */
/* Returns 0, or -1 if an integer dot left the int32 range.                  */
/* ------------------------------------------------------------------------- */
int zo_sgd_epoch_e2e(const uint8_t *codes1, const uint8_t *codes2, const float *levels,
                     const uint16_t *grid_idx, float grid_lo, float grid_step, const float *b,
                     int64_t n, int64_t d, int bits, float *x, int64_t batch, float lr,
                     int grad_bits, int model_bits, uint64_t seed, uint32_t epoch,
                     int64_t first_step, int64_t num_steps, int32_t *dbg_m, int32_t *dbg_acc,
                     float *dbg_r, float *dbg_g, int32_t *dbg_gq)
{
    int K = 1 << bits;
    int32_t *m = malloc(sizeof(int32_t) * (size_t)d);
    int32_t *gq = malloc(sizeof(int32_t) * (size_t)d);
    float *r = malloc(sizeof(float) * (size_t)batch);
    float *g = malloc(sizeof(float) * (size_t)d);
    int64_t *acc = malloc(sizeof(int64_t) * (size_t)batch);
    int rc = 0;
    if (num_steps < 0) num_steps = n / batch - first_step;
    for (int64_t t = first_step; t < first_step + num_steps; ++t) {
        const uint8_t *c1 = codes1 + t * batch * d, *c2 = codes2 + t * batch * d;
        const float *bb = b + t * batch;
        /* Q3: quantise the model (Supp. C) */
        float sigma = zo_quantize_vec(x, d, model_bits, seed, epoch, (uint64_t)t, 3, m);
        int64_t summ = 0;
        for (int64_t j = 0; j < d; ++j) summ += m[j];
        /* dot pass on copy 2 with the quantised model */
        for (int64_t i = 0; i < batch; ++i) {
            int64_t a = 0;
            for (int64_t j = 0; j < d; ++j)
                a += (int64_t)grid_idx[j * K + c2[i * d + j]] * (int64_t)m[j];
            if (a > INT32_MAX || a < INT32_MIN) rc = -1;
            acc[i] = a;
            double z = (double)sigma *
                       ((double)grid_lo * (double)summ + (double)grid_step * (double)a);
            r[i] = (float)z - bb[i];
        }
        /* gradient pass on copy 1: the mean over the batch of Q1(a_i) r_i, summed in fp64 in
         * sample order (each product is exact) and rounded to fp32 once */
        for (int64_t j = 0; j < d; ++j) {
            double sum = 0.0;
            for (int64_t i = 0; i < batch; ++i)
                sum += (double)levels[j * K + c1[i * d + j]] * (double)r[i];
            g[j] = (float)(sum / (double)batch);
        }
        /* Q4: quantise the gradient (Supp. D), then full-precision update */
        if (grad_bits > 0) {
            float sg = zo_quantize_vec(g, d, grad_bits, seed, epoch, (uint64_t)t, 4, gq);
            for (int64_t j = 0; j < d; ++j) {
                float gh = sg * (float)gq[j];
                float step = lr * gh;
                x[j] = x[j] - step;
            }
        } else {
            for (int64_t j = 0; j < d; ++j) {
                float step = lr * g[j];
                x[j] = x[j] - step;
            }
        }
        if (t == first_step + num_steps - 1) {
            if (dbg_m) memcpy(dbg_m, m, sizeof(int32_t) * (size_t)d);
            if (dbg_acc) for (int64_t i = 0; i < batch; ++i) dbg_acc[i] = (int32_t)acc[i];
            if (dbg_r) memcpy(dbg_r, r, sizeof(float) * (size_t)batch);
            if (dbg_g) memcpy(dbg_g, g, sizeof(float) * (size_t)d);
            if (dbg_gq && grad_bits > 0) memcpy(dbg_gq, gq, sizeof(int32_t) * (size_t)d);
        }
    }
    free(m); free(gq); free(r); free(g); free(acc);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Loss  F(x) = 1/(2n) sum_i (a_i^T x - b_i)^2  (Sec. 1 eq. (1) with the     */
/* square loss), fp64.                                                       */
/* ------------------------------------------------------------------------- */
double zo_loss(const float *A, int64_t n, int64_t d, int64_t lda, const float *b, const float *x)
{
    double F = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double z = 0.0;
        for (int64_t j = 0; j < d; ++j) z += (double)A[i * lda + j] * (double)x[j];
        double r = z - (double)b[i];
        F += r * r;
    }
    return F / (2.0 * (double)n);
}

/* The same with a_ij replaced by the decoded levels of one quantised copy. */
double zo_loss_codes(const uint8_t *codes, const float *levels, int bits, int64_t n, int64_t d,
                     const float *b, const float *x)
{
    int K = 1 << bits;
    double F = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double z = 0.0;
        for (int64_t j = 0; j < d; ++j)
            z += (double)levels[j * K + codes[i * d + j]] * (double)x[j];
        double r = z - (double)b[i];
        F += r * r;
    }
    return F / (2.0 * (double)n);
}
