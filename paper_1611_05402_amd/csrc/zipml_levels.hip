// zipml_levels: per-feature ranges and quantisation levels.
//
// Supp. A.3 "Column Scaling": one range per feature from the column minimum and maximum.
// Sec. 2.1: uniform levels.  Sec. 3.1-3.2: variance-optimal levels -- one scan of the data into
// M equal bins per feature (count, sum, sum of squares of the normalised values), then the dynamic
// program T(k,m) = min_j T(k-1,j) + V(j,m) over the bin edges -- on the device (one workgroup per
// feature, k_dp_levels) when its tables fit in LDS, else on the host cores; optionally over the
// candidates that a greedy merge of the bins leaves (Sec. 3.2; supplement, Algorithm 1).
#include "zipml_device.h"
#include "zipml_host.h"

#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <limits>
#include <thread>
#include <vector>

namespace zipml {

// Order-preserving map float -> uint32 so that min/max can use integer atomics.
__device__ __forceinline__ uint32_t f2key(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key2f(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7FFFFFFFu) : ~k);
}

__global__ void k_range_init(uint32_t *kmin, uint32_t *kmax, int64_t d)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j < d) { kmin[j] = 0xFFFFFFFFu; kmax[j] = 0u; }
}

// One thread per feature (consecutive lanes read consecutive floats of a row), a slab of rows per
// blockIdx.y.
__global__ __launch_bounds__(256) void k_range_scan(const float *__restrict__ A, int64_t n,
                                                    int64_t d, int64_t lda, int64_t rows_per_slab,
                                                    uint32_t *kmin, uint32_t *kmax)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= d) return;
    const int64_t i0 = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t i1 = i0 + rows_per_slab < n ? i0 + rows_per_slab : n;
    if (i0 >= i1) return;
    float mn = A[i0 * lda + j], mx = mn;
    for (int64_t i = i0 + 1; i < i1; ++i) {
        const float v = A[i * lda + j];
        mn = v < mn ? v : mn;
        mx = v > mx ? v : mx;
    }
    atomicMin(kmin + j, f2key(mn));
    atomicMax(kmax + j, f2key(mx));
}

__global__ void k_range_final(const uint32_t *kmin, const uint32_t *kmax, int64_t d, int symmetric,
                              float *lo, float *hi)
{
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= d) return;
    float mn = key2f(kmin[j]), mx = key2f(kmax[j]);
    if (symmetric) {
        const float m = fabsf(mn) > fabsf(mx) ? fabsf(mn) : fabsf(mx);
        mn = -m;
        mx = m;
    }
    lo[j] = mn;
    hi[j] = mx;
}

// L[j][c] = fp32( lo + c (hi - lo) / (K - 1) ), evaluated in fp64; grid index = c.
__global__ void k_levels_uniform(const float *__restrict__ lo, const float *__restrict__ hi,
                                 int64_t d, int K, float *__restrict__ levels,
                                 uint16_t *__restrict__ grid)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= d * K) return;
    const int64_t j = e / K;
    const int c = (int)(e % K);
    const double l = (double)lo[j], w = (double)hi[j] - (double)lo[j];
    levels[e] = (float)(l + ((double)c * w) / (double)(K - 1));
    if (grid) grid[e] = (uint16_t)c;
}

__global__ void k_zero_f64(double *p, int64_t count)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.0;
}

// Per-bin moments of the normalised values; hist is [d][M][3] fp64 (count, sum t, sum t^2).
// One atomic per value and moment straight to memory ran at the rate the memory side takes
// atomics (about 22 per ns: 18-28 ms for 65,536 x 2048 values).  Here a workgroup owns F
// consecutive features -- as many as have their M bins in LDS, F a divisor of 256 -- and a slab
// of rows (all rows when the blocks of features fill the device), adds into LDS, and sends its
// bins to memory once at the end: 0.44 ms for the same matrix.  The counts are 32-bit integers
// to save LDS; the two sums are fp64.
__global__ __launch_bounds__(256) void k_hist(const float *__restrict__ A, int64_t n, int64_t d,
                                              int64_t lda, int64_t rows_per_slab,
                                              const float *__restrict__ lo,
                                              const float *__restrict__ hi, int M, int F,
                                              int direct, double *__restrict__ hist)
{
    extern __shared__ __align__(16) unsigned char hist_smem[];
    double *sh = (double *)hist_smem;                        // [F][M][2] sum t, sum t^2
    uint32_t *cnt = (uint32_t *)(sh + (size_t)F * M * 2);    // [F][M] counts (a slab has fewer than 2^32 rows)
    const int tid = threadIdx.x;
    // Blocks go round the 8 dies in turn, and neighbouring blocks of features share the cache
    // lines of every row: block b takes features block (b % 8) * (gridDim.x / 8) + b / 8, so that
    // neighbours run on one die at about the same time.  (gridDim.x is a multiple of 8; blocks
    // past the last features block leave.)
    const int64_t fb = (int64_t)(blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    const int64_t j0 = fb * F;
    if (j0 >= d) return;
    const int nf = (int)(d - j0 < F ? d - j0 : F);
    const int64_t i0 = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t i1 = i0 + rows_per_slab < n ? i0 + rows_per_slab : n;
    for (int e = tid; e < nf * M * 2; e += 256) sh[e] = 0.0;
    for (int e = tid; e < nf * M; e += 256) cnt[e] = 0u;
    __syncthreads();
    // F divides 256: thread t keeps feature t % F for good (its range in registers) and takes the
    // rows t / F, t / F + 256 / F, ...  Sixteen values are requested before the first is used, with
    // loads that no branch can skip (rows past the slab repeat its last row and are not counted):
    // a load behind a branch makes the compiler wait for it on the spot, and one workgroup per
    // compute unit has nothing else to hide that latency with.  Nothing in the loop reads LDS, so
    // the additions are never waited for.
    const int f = tid % F;
    const bool live_col = f < nf;
    if (i0 < i1 && live_col) {
        constexpr int U = 16;
        const int rows_step = 256 / F;
        const double l = (double)lo[j0 + f], w = (double)hi[j0 + f] - (double)lo[j0 + f];
        const float *col = A + j0 + f;
        double *hf = sh + (size_t)f * M * 2;
        uint32_t *cf = cnt + (size_t)f * M;
        for (int64_t i = i0 + tid / F; i < i1; i += (int64_t)U * rows_step) {
            float a[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t r = i + (int64_t)u * rows_step;
                a[u] = col[(r < i1 ? r : i1 - 1) * lda];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i + (int64_t)u * rows_step < i1) {
                    double t = 0.0;
                    if (w > 0.0) {
                        t = ((double)a[u] - l) / w;
                        t = t < 0.0 ? 0.0 : t;
                        t = t > 1.0 ? 1.0 : t;
                    }
                    int m = (int)(t * (double)M);
                    if (m > M - 1) m = M - 1;
                    atomicAdd(cf + m, 1u);
                    unsafeAtomicAdd(hf + 2 * m, t);
                    unsafeAtomicAdd(hf + 2 * m + 1, t * t);
                }
            }
        }
    }
    __syncthreads();
    double *out = hist + (size_t)j0 * M * 3;
    for (int e = tid; e < nf * M * 3; e += 256) {
        const int bin = e / 3, c = e % 3;
        const double v = c == 0 ? (double)cnt[bin] : sh[bin * 2 + c - 1];
        if (direct) out[e] = v;                      // the only slab: nobody else adds to these bins
        else if (v != 0.0) unsafeAtomicAdd(out + e, v);
    }
}
// Features per workgroup of k_hist and its LDS bytes.
inline int hist_features(int M, int lds_limit)
{
    const int f = (int)(((size_t)lds_limit - 1024) / ((size_t)M * 20 + 16));
    return f < 1 ? 1 : f > 32 ? 32 : f;
}
inline size_t hist_lds_bytes(int M, int F) { return (size_t)F * ((size_t)M * 20 + 16); }

// ---------------------------------------------------------------------------------------------
// Host dynamic program for one feature: s intervals over the M+1 bin edges m/M.
// Returns the total variance; idx[0..s] are the chosen edges.  Ties: smallest j.
// ---------------------------------------------------------------------------------------------
// The dynamic program of Sec. 3 on the device: one workgroup per feature, everything in LDS.
//   T(1, m) = V(0, m),  T(k, m) = min_{k-1 <= j <= m-1} T(k-1, j) + V(j, m),
//   V(j, m) = sum over the points in [d_j, d_m) of (d_m - t)(t - d_j), from prefix moments.
// The arithmetic is that of the host version below, operation by operation (prefix sums in index
// order, the same expression for V, the smallest j on ties), so both give the same levels.
// Thread tid takes the end points m = tid, tid + 256, ...; in step i of the inner loop all threads
// read the same j, which LDS serves as a broadcast.
// LDS: 6 arrays of M+1 doubles and the argmin table (s+1) x (M+1) uint16.
__host__ __device__ inline size_t dp_lds_bytes(int M, int s)
{
    const size_t W = (size_t)M + 1;
    return 6 * W * sizeof(double) + (((size_t)s + 1) * W * sizeof(uint16_t) + 15) / 16 * 16 + 64;
}
// With sel / count (the greedy search below): the candidates of feature j are the count[j] + 1 bin
// edges sel[j][0 .. count[j]] and hist holds the moments of the intervals between them; Mcap is
// the largest number of intervals a feature can have (it sizes the tables).
__global__ __launch_bounds__(256) void k_dp_levels(const double *__restrict__ hist,
                                                   const float *__restrict__ lo,
                                                   const float *__restrict__ hi, int64_t d, int Mgrid,
                                                   int s, float *__restrict__ levels,
                                                   uint16_t *__restrict__ grid,
                                                   double *__restrict__ objective,
                                                   const uint16_t *__restrict__ sel,
                                                   const int *__restrict__ count, int Mcap)
{
    extern __shared__ __align__(16) unsigned char dp_smem[];
    const int K = s + 1, tid = threadIdx.x;
    const int Wcap = Mcap + 1;
    double *C = (double *)dp_smem, *S1 = C + Wcap, *S2 = S1 + Wcap, *edge = S2 + Wcap,
           *prev = edge + Wcap, *cur = prev + Wcap;
    uint16_t *arg = (uint16_t *)(dp_smem + 6 * (size_t)Wcap * sizeof(double));   // [s+1][W]
    const double INF = __longlong_as_double(0x7FF0000000000000ll);
    for (int64_t j = blockIdx.x; j < d; j += gridDim.x) {
        const double *mom = hist + (size_t)j * Mgrid * 3;
        const uint16_t *cand = sel ? sel + (size_t)j * (Mgrid + 1) : nullptr;
        const int M = sel ? count[j] : Mgrid;
        const int W = M + 1;
        prev = edge + Wcap;
        cur = prev + Wcap;
        __syncthreads();
        // prefix moments, in index order (three chains, one thread each)
        if (tid < 3) {
            double *dst = tid == 0 ? C : tid == 1 ? S1 : S2;
            double acc = 0.0;
            dst[0] = 0.0;
            for (int m = 0; m < M; ++m) {
                acc = acc + mom[m * 3 + tid];
                dst[m + 1] = acc;
            }
        }
        for (int m = tid; m < W; m += 256) {
            edge[m] = (double)(cand ? (int)cand[m] : m) / (double)Mgrid;
            prev[m] = INF;
        }
        __syncthreads();
        auto V = [&](int jj, int m) {
            const double dj = edge[jj], dm = edge[m];
            return -(S2[m] - S2[jj]) + (dj + dm) * (S1[m] - S1[jj]) - dj * dm * (C[m] - C[jj]);
        };
        for (int m = 1 + tid; m <= M; m += 256) {
            prev[m] = V(0, m);
            arg[1 * W + m] = 0;
        }
        __syncthreads();
        for (int k = 2; k <= s; ++k) {
            for (int m = tid; m < W; m += 256) {
                double best = INF;
                int bj = k - 1;
                if (m >= k) {
                    // (this end point's own terms stay in registers; four j at a time, so that the
                    // LDS reads of one are in flight while the arithmetic of another runs)
                    const double dm = edge[m], s2m = S2[m], s1m = S1[m], cm = C[m];
#pragma unroll 4
                    for (int jj = k - 1; jj <= m - 1; ++jj) {
                        const double dj = edge[jj];
                        const double vjm = -(s2m - S2[jj]) + (dj + dm) * (s1m - S1[jj]) - dj * dm * (cm - C[jj]);
                        const double v = prev[jj] + vjm;
                        if (v < best) { best = v; bj = jj; }
                    }
                    arg[(size_t)k * W + m] = (uint16_t)bj;
                }
                cur[m] = best;
            }
            __syncthreads();
            double *t = prev; prev = cur; cur = t;
        }
        if (tid == 0) {
            const double total = prev[M];
            double cnt = C[M];
            objective[j] = cnt > 0.0 ? total / cnt : 0.0;
            const double l = (double)lo[j], w = (double)hi[j] - l;
            int m = M;
            for (int k = s; k >= 1; --k) {
                const int g = cand ? (int)cand[m] : m;
                if (grid) grid[(size_t)j * K + k] = (uint16_t)g;
                levels[(size_t)j * K + k] = (float)(l + (w * (double)g) / (double)Mgrid);
                m = arg[(size_t)k * W + m];
            }
            if (grid) grid[(size_t)j * K] = 0;
            levels[(size_t)j * K] = (float)(l + (w * 0.0) / (double)Mgrid);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Greedy merging of intervals (supplement, "A Greedy Algorithm for Finding Quantization Points",
// Algorithm 1, with gamma = 1 and delta = 1), on the M bins of the candidate grid: one workgroup
// per feature, the partition and the moments of its intervals in LDS.  While more than 4k + 1
// intervals are left, consecutive intervals are paired up (an odd one at the end stays), every
// pair gets the error of the merged interval [a, b], -S2 + (a + b) S1 - a b S0, from the sum of
// the two intervals' moments; the 2k pairs with the largest error (equal errors: further left
// first) stay split, the others are merged.  The end points that are left become the candidates
// of the dynamic program (Sec. 3.2): the moments of the intervals replace the feature's bin
// moments in place, sel[j][0 .. count[j]] are the bin edges.
// Every pair's rank is found by counting (no sort: the order of equal errors is part of the
// result); the partition is compacted in place, 256 pairs at a time: a pair's new position is
// never behind its old one, so a block of pairs that has been read can be written before the
// next block is read.
__host__ __device__ inline size_t greedy_lds_bytes(int M)
{
    return (size_t)M * 3 * sizeof(double) + ((size_t)M / 2 + 2) * sizeof(double) +
           ((size_t)M + 2 + 2 * ((size_t)M / 2 + 2)) * sizeof(int) + 64;
}
__global__ __launch_bounds__(256) void k_greedy_intervals(double *__restrict__ hist, int64_t d, int M,
                                                          int k, uint16_t *__restrict__ sel,
                                                          int *__restrict__ count)
{
    extern __shared__ __align__(16) unsigned char gr_smem[];
    const int tid = threadIdx.x;
    double *mom = (double *)gr_smem;                 // [M][3]
    double *e = mom + (size_t)M * 3;                 // [M/2 + 2]
    int *edge = (int *)(e + M / 2 + 2);              // [M + 2]
    int *keep = edge + M + 2;                        // [M/2 + 2]
    int *offs = keep + M / 2 + 2;                    // [M/2 + 2]
    const int q = 2 * k, limit = 4 * k + 1;
    for (int64_t j = blockIdx.x; j < d; j += gridDim.x) {
        double *h = hist + (size_t)j * M * 3;
        __syncthreads();
        for (int m = tid; m < M * 3; m += 256) mom[m] = h[m];
        for (int m = tid; m <= M; m += 256) edge[m] = m;
        __syncthreads();
        int P = M;
        while (P > limit) {
            const int pairs = P / 2;
            for (int i = tid; i < pairs; i += 256) {
                const double a = (double)edge[2 * i] / (double)M, b = (double)edge[2 * i + 2] / (double)M;
                const double s0 = mom[(2 * i) * 3 + 0] + mom[(2 * i + 1) * 3 + 0];
                const double s1 = mom[(2 * i) * 3 + 1] + mom[(2 * i + 1) * 3 + 1];
                const double s2 = mom[(2 * i) * 3 + 2] + mom[(2 * i + 1) * 3 + 2];
                e[i] = -s2 + (a + b) * s1 - a * b * s0;
            }
            __syncthreads();
            for (int i = tid; i < pairs; i += 256) {
                const double ei = e[i];
                int before = 0;
                for (int jj = 0; jj < pairs; ++jj) {
                    const double ej = e[jj];
                    before += (ej > ei || (ej == ei && jj < i)) ? 1 : 0;
                }
                keep[i] = before < q ? 1 : 0;
            }
            __syncthreads();
            if (tid == 0) {
                int out = 0;
                for (int i = 0; i < pairs; ++i) { offs[i] = out; out += keep[i] ? 2 : 1; }
                offs[pairs] = out;
            }
            __syncthreads();
            const int odd = P & 1;
            // the odd interval at the end: taken out before anything is overwritten
            const int last_edge = edge[P - 1];
            const double l0 = mom[(P - 1) * 3 + 0], l1 = mom[(P - 1) * 3 + 1], l2 = mom[(P - 1) * 3 + 2];
            const int newP = offs[pairs] + odd;
            __syncthreads();
            for (int base = 0; base < pairs; base += 256) {
                const int i = base + tid;
                int e0 = 0, e1 = 0, kp = 0, o = 0;
                double a0 = 0, a1 = 0, a2 = 0, b0 = 0, b1 = 0, b2 = 0;
                if (i < pairs) {
                    e0 = edge[2 * i]; e1 = edge[2 * i + 1]; kp = keep[i]; o = offs[i];
                    a0 = mom[(2 * i) * 3 + 0]; a1 = mom[(2 * i) * 3 + 1]; a2 = mom[(2 * i) * 3 + 2];
                    b0 = mom[(2 * i + 1) * 3 + 0]; b1 = mom[(2 * i + 1) * 3 + 1]; b2 = mom[(2 * i + 1) * 3 + 2];
                }
                __syncthreads();
                if (i < pairs) {
                    if (kp) {
                        edge[o] = e0; edge[o + 1] = e1;
                        mom[o * 3 + 0] = a0; mom[o * 3 + 1] = a1; mom[o * 3 + 2] = a2;
                        mom[(o + 1) * 3 + 0] = b0; mom[(o + 1) * 3 + 1] = b1; mom[(o + 1) * 3 + 2] = b2;
                    } else {
                        edge[o] = e0;
                        mom[o * 3 + 0] = a0 + b0; mom[o * 3 + 1] = a1 + b1; mom[o * 3 + 2] = a2 + b2;
                    }
                }
            }
            __syncthreads();
            if (tid == 0) {
                if (odd) {
                    const int o = newP - 1;
                    edge[o] = last_edge;
                    mom[o * 3 + 0] = l0; mom[o * 3 + 1] = l1; mom[o * 3 + 2] = l2;
                }
                edge[newP] = M;
            }
            __syncthreads();
            P = newP;
        }
        for (int m = tid; m < P * 3; m += 256) h[m] = mom[m];
        for (int m = tid; m <= P; m += 256) sel[(size_t)j * (M + 1) + m] = (uint16_t)edge[m];
        if (tid == 0) count[j] = P;
    }
}

static double dp_one_feature(const double *mom, int M, int s, std::vector<double> &C,
                             std::vector<double> &S1, std::vector<double> &S2,
                             std::vector<double> &prev, std::vector<double> &cur,
                             std::vector<uint16_t> &arg, int *idx)
{
    const size_t W = (size_t)M + 1;
    C[0] = S1[0] = S2[0] = 0.0;
    for (int m = 0; m < M; ++m) {
        C[m + 1] = C[m] + mom[m * 3 + 0];
        S1[m + 1] = S1[m] + mom[m * 3 + 1];
        S2[m + 1] = S2[m] + mom[m * 3 + 2];
    }
    auto edge = [&](int m) { return (double)m / (double)M; };   // M need not be a power of two
    auto V = [&](int j, int m) {
        const double dj = edge(j), dm = edge(m);
        return -(S2[m] - S2[j]) + (dj + dm) * (S1[m] - S1[j]) - dj * dm * (C[m] - C[j]);
    };
    const double INF = std::numeric_limits<double>::infinity();
    std::fill(prev.begin(), prev.end(), INF);
    for (int m = 1; m <= M; ++m) { prev[m] = V(0, m); arg[1 * W + m] = 0; }
    for (int k = 2; k <= s; ++k) {
        std::fill(cur.begin(), cur.end(), INF);
        for (int m = k; m <= M; ++m) {
            double best = INF;
            int bj = k - 1;
            for (int j = k - 1; j <= m - 1; ++j) {
                const double v = prev[j] + V(j, m);
                if (v < best) { best = v; bj = j; }
            }
            cur[m] = best;
            arg[(size_t)k * W + m] = (uint16_t)bj;
        }
        std::swap(prev, cur);
    }
    const double total = prev[M];
    int m = M;
    for (int k = s; k >= 1; --k) { idx[k] = m; m = arg[(size_t)k * W + m]; }
    idx[0] = 0;
    return total;
}

static size_t levels_workspace_bytes(int64_t d, int n_candidates)
{
    size_t keys = (size_t)round_up(d * 8, 256);
    size_t hist = (size_t)d * (size_t)n_candidates * 3 * sizeof(double);
    size_t objective = (size_t)d * sizeof(double);     // per-feature value of the dynamic program
    // candidates left by the greedy search: bin edges [d][n_candidates + 1] uint16, their number [d]
    size_t greedy = n_candidates > 0 ? (size_t)round_up(d * ((int64_t)n_candidates + 1) * 2, 256) + (size_t)d * 4 : 0;
    return keys + hist + objective + greedy;
}

}  // namespace zipml

using namespace zipml;

extern "C" size_t zipml_workspace_bytes(int64_t n, int64_t d, int bits, int64_t batch,
                                        int n_candidates)
{
    if (n <= 0 || d <= 0 || !valid_bits(bits) || batch <= 0 || n_candidates < 0) return 0;
    size_t sgd = Workspace::xchg_offset(d, batch) + Workspace::xchg_bytes(d, batch);
    size_t lev = levels_workspace_bytes(d, n_candidates);
    size_t loss = (2048 + 1) * sizeof(double) + 1024;   // partial sums, result, flags of the level check
    size_t need = std::max(sgd, std::max(lev, loss));
    return (size_t)round_up((int64_t)need, 256);
}

extern "C" int zipml_levels(void *stream, const float *A_dev, int64_t n, int64_t d, int64_t lda,
                            int bits, int mode, int flags, int n_candidates, float *lo_dev,
                            float *hi_dev, float *levels_dev, uint16_t *grid_idx_dev,
                            double *mean_variance_host, void *workspace_dev,
                            size_t workspace_bytes)
{
    if (!lo_dev || !hi_dev || !levels_dev || d <= 0 || !valid_bits(bits)) return ZIPML_EINVAL;
    if (mode != ZIPML_UNIFORM && mode != ZIPML_OPTIMAL && mode != ZIPML_GREEDY) return ZIPML_EINVAL;
    const bool search = mode == ZIPML_OPTIMAL || mode == ZIPML_GREEDY;
    if (flags & ~(ZIPML_RANGE_GIVEN | ZIPML_SYMMETRIC)) return ZIPML_EINVAL;
    const bool need_data = !(flags & ZIPML_RANGE_GIVEN) || search;
    if (need_data && (!A_dev || n <= 0 || lda < d)) return ZIPML_EINVAL;
    const int K = 1 << bits;
    if (search && (n_candidates < K - 1 || n_candidates > 4096)) return ZIPML_EINVAL;
    if (!aligned16(lo_dev) || !aligned16(hi_dev) || !aligned16(levels_dev) ||
        (grid_idx_dev && !aligned16(grid_idx_dev)) || (A_dev && (reinterpret_cast<uintptr_t>(A_dev) & 3u)))
        return ZIPML_EALIGN;
    const size_t need = levels_workspace_bytes(d, search ? n_candidates : 0);
    if (need_data && (!workspace_dev || workspace_bytes < need || !aligned16(workspace_dev)))
        return ZIPML_EWORKSPACE;
    hipStream_t s = entry_stream(stream);
    const unsigned cb = (unsigned)((d + 255) / 256);
    // rows are split into slabs so that the scan fills the device
    int64_t slabs = std::max<int64_t>(1, std::min<int64_t>(n / 64 + 1, 4096 / cb + 1));
    const int64_t rows_per_slab = n > 0 ? (n + slabs - 1) / slabs : 1;
    slabs = n > 0 ? (n + rows_per_slab - 1) / rows_per_slab : 1;

    if (!(flags & ZIPML_RANGE_GIVEN)) {
        uint32_t *kmin = (uint32_t *)workspace_dev, *kmax = kmin + d;
        hipLaunchKernelGGL(k_range_init, dim3(cb), dim3(256), 0, s, kmin, kmax, d);
        hipLaunchKernelGGL(k_range_scan, dim3(cb, (unsigned)slabs), dim3(256), 0, s, A_dev, n, d, lda,
                           rows_per_slab, kmin, kmax);
        hipLaunchKernelGGL(k_range_final, dim3(cb), dim3(256), 0, s, kmin, kmax, d,
                           (flags & ZIPML_SYMMETRIC) ? 1 : 0, lo_dev, hi_dev);
        if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    }
    if (mode == ZIPML_UNIFORM) {
        const int64_t total = d * K;
        hipLaunchKernelGGL(k_levels_uniform, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                           lo_dev, hi_dev, d, K, levels_dev, grid_idx_dev);
        return hip_check(hipGetLastError());
    }

    // ---- OPTIMAL / GREEDY: bin moments on the device, then the dynamic program (device or host, below)
    const int M = n_candidates, sI = K - 1;
    double *hist_dev = (double *)((unsigned char *)workspace_dev + round_up(d * 8, 256));
    const int64_t hcount = d * (int64_t)M * 3;
    hipLaunchKernelGGL(k_zero_f64, dim3((unsigned)((hcount + 255) / 256)), dim3(256), 0, s, hist_dev,
                       hcount);
    int lds_limit = 0, dev = 0;
    if (HIP_FAILED(hipGetDevice(&dev)) ||
        HIP_FAILED(hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev)))
        return ZIPML_ELAUNCH;
    {
        // Blocks of F features, each with all rows when that fills the device (no additions in
        // memory at all then: with slabs, the workgroups' additions of their bins to memory cost
        // more than the scan); F is the largest number of features that keeps the number of
        // rounds of workgroups times F smallest.  Few features: slabs of rows as well.
        int cus = 0;
        if (HIP_FAILED(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev))) return ZIPML_ELAUNCH;
        const int Fmax = hist_features(M, lds_limit);
        int F = 1;
        int64_t best = -1;
        for (int f = 1; f <= Fmax; f *= 2) {      // (F divides 256)
            const int64_t rounds = ((d + f - 1) / f + cus - 1) / cus;
            if (best < 0 || rounds * f <= best) { best = rounds * f; F = f; }
        }
        // development override: a power of two that fits
        if (const long long v = knob(ZIPML_KNOB_HIST_FEATURES); v >= 1 && v <= Fmax && (v & (v - 1)) == 0) F = (int)v;
        const size_t hl = hist_lds_bytes(M, F);
        if (hl > (size_t)lds_limit) return ZIPML_EUNSUPPORTED;
        const int64_t fblocks = (d + F - 1) / F;
        int64_t hs = fblocks >= cus ? 1 : std::max<int64_t>(1, std::min<int64_t>((n + 255) / 256, (2 * cus + fblocks - 1) / fblocks));
        const int64_t hrows = (n + hs - 1) / hs;
        hs = (n + hrows - 1) / hrows;
        if (fblocks > 0x7fffffff || hs > 65535) return ZIPML_EINVAL;
        if (HIP_FAILED(hipFuncSetAttribute((const void *)k_hist, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)hl)))
            return ZIPML_ELAUNCH;
        hipLaunchKernelGGL(k_hist, dim3((unsigned)round_up(fblocks, 8), (unsigned)hs), dim3(256), hl, s, A_dev, n, d, lda,
                           hrows, lo_dev, hi_dev, M, F, hs == 1 ? 1 : 0, hist_dev);
        if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    }

    // The dynamic program runs on the device when its tables fit in LDS (up to 5 bits at 1024
    // candidates), else on the host cores.
    // GREEDY: the greedy search leaves at most 4 (K - 1) + 1 intervals per feature, whose end points
    // are the candidates of the dynamic program; with no more bins than that nothing is merged and
    // the search is the plain one.  Both steps run on the device (no host version).
    const int Mcap = 4 * sI + 1;
    const bool greedy = mode == ZIPML_GREEDY && M > Mcap;
    const size_t dp_lds = greedy ? dp_lds_bytes(Mcap, sI) : dp_lds_bytes(M, sI);
    if (greedy && (dp_lds > (size_t)lds_limit || greedy_lds_bytes(M) > (size_t)lds_limit))
        return ZIPML_EUNSUPPORTED;
    if (greedy || (dp_lds <= (size_t)lds_limit && knob(ZIPML_KNOB_HOST_DP) <= 0)) {
        double *objective_dev = hist_dev + hcount;
        uint16_t *grid_dev = grid_idx_dev;       // may be null
        uint16_t *sel_dev = nullptr;
        int *count_dev = nullptr;
        const unsigned blocks = (unsigned)(d < 2048 ? d : 2048);
        if (greedy) {
            sel_dev = (uint16_t *)(objective_dev + d);
            count_dev = (int *)((unsigned char *)sel_dev + round_up(d * ((int64_t)M + 1) * 2, 256));
            const size_t gr_lds = greedy_lds_bytes(M);
            if (HIP_FAILED(hipFuncSetAttribute((const void *)k_greedy_intervals,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)gr_lds)))
                return ZIPML_ELAUNCH;
            hipLaunchKernelGGL(k_greedy_intervals, dim3(blocks), dim3(256), gr_lds, s, hist_dev, d, M, sI,
                               sel_dev, count_dev);
            if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
        }
        if (HIP_FAILED(hipFuncSetAttribute((const void *)k_dp_levels,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)dp_lds)))
            return ZIPML_ELAUNCH;
        hipLaunchKernelGGL(k_dp_levels, dim3(blocks), dim3(256), dp_lds, s, hist_dev, lo_dev, hi_dev, d,
                           M, sI, levels_dev, grid_dev, objective_dev, (const uint16_t *)sel_dev,
                           (const int *)count_dev, greedy ? Mcap : M);
        if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
        if (mean_variance_host) {
            std::vector<double> per_feature((size_t)d);
            if (hipMemcpyAsync(per_feature.data(), objective_dev, sizeof(double) * (size_t)d,
                               hipMemcpyDeviceToHost, s) != hipSuccess ||
                hipStreamSynchronize(s) != hipSuccess)
                return ZIPML_ELAUNCH;
            double mv = 0.0;
            for (int64_t j = 0; j < d; ++j) mv += per_feature[(size_t)j];
            *mean_variance_host = mv / (double)d;
        }
        return ZIPML_OK;
    }
    std::vector<double> hist((size_t)hcount);
    std::vector<float> lo((size_t)d), hi((size_t)d);
    if (hipMemcpyAsync(hist.data(), hist_dev, sizeof(double) * (size_t)hcount, hipMemcpyDeviceToHost,
                       s) != hipSuccess ||
        hipMemcpyAsync(lo.data(), lo_dev, sizeof(float) * (size_t)d, hipMemcpyDeviceToHost, s) !=
            hipSuccess ||
        hipMemcpyAsync(hi.data(), hi_dev, sizeof(float) * (size_t)d, hipMemcpyDeviceToHost, s) !=
            hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return ZIPML_ELAUNCH;

    std::vector<float> levels((size_t)d * K);
    std::vector<uint16_t> grid((size_t)d * K);
    std::vector<double> per_feature((size_t)d, 0.0);
    unsigned nthreads = std::max(1u, std::min(std::thread::hardware_concurrency(), 16u));
    if ((int64_t)nthreads > d) nthreads = (unsigned)d;
    std::atomic<int64_t> next{0};
    auto worker = [&]() {
        const size_t W = (size_t)M + 1;
        std::vector<double> C(W), S1(W), S2(W), prev(W), cur(W);
        std::vector<uint16_t> arg(W * ((size_t)sI + 1));
        std::vector<int> idx((size_t)sI + 1);
        for (;;) {
            const int64_t j = next.fetch_add(1);
            if (j >= d) break;
            const double *mom = hist.data() + (size_t)j * M * 3;
            const double total = dp_one_feature(mom, M, sI, C, S1, S2, prev, cur, arg, idx.data());
            double cnt = 0.0;
            for (int m = 0; m < M; ++m) cnt += mom[m * 3];
            per_feature[(size_t)j] = cnt > 0.0 ? total / cnt : 0.0;
            const double l = (double)lo[(size_t)j], w = (double)hi[(size_t)j] - l;
            for (int c = 0; c < K; ++c) {
                grid[(size_t)j * K + c] = (uint16_t)idx[c];
                levels[(size_t)j * K + c] = (float)(l + (w * (double)idx[c]) / (double)M);
            }
        }
    };
    std::vector<std::thread> pool;
    for (unsigned t = 1; t < nthreads; ++t) pool.emplace_back(worker);
    worker();
    for (auto &t : pool) t.join();
    if (mean_variance_host) {
        double mv = 0.0;
        for (int64_t j = 0; j < d; ++j) mv += per_feature[(size_t)j];
        *mean_variance_host = mv / (double)d;
    }
    if (hipMemcpyAsync(levels_dev, levels.data(), sizeof(float) * levels.size(),
                       hipMemcpyHostToDevice, s) != hipSuccess)
        return ZIPML_ELAUNCH;
    if (grid_idx_dev && hipMemcpyAsync(grid_idx_dev, grid.data(), sizeof(uint16_t) * grid.size(),
                                       hipMemcpyHostToDevice, s) != hipSuccess)
        return ZIPML_ELAUNCH;
    if (hipStreamSynchronize(s) != hipSuccess) return ZIPML_ELAUNCH;
    return ZIPML_OK;
}

extern "C" int zipml_debug_set(int knob_id, int64_t value)
{
    if (knob_id < 0 || knob_id >= ZIPML_KNOB_COUNT || value < -1) return ZIPML_EINVAL;
    g_knob[knob_id].store((long long)value + 1, std::memory_order_relaxed);
    return ZIPML_OK;
}

extern "C" const char *zipml_strerror(int code)
{
    switch (code) {
        case ZIPML_OK: return "ok";
        case ZIPML_EINVAL: return "invalid argument";
        case ZIPML_EALIGN: return "device pointer not 16-byte aligned";
        case ZIPML_ERANGE: return "integer dot product could overflow int32";
        case ZIPML_EWORKSPACE: return "workspace missing or too small";
        case ZIPML_ELAUNCH: return "HIP launch or copy failed";
        case ZIPML_EUNSUPPORTED: return "not supported by this build";
        case ZIPML_ETIMEOUT: return "grid-wide wait timed out";
        default: return "unknown error";
    }
}
