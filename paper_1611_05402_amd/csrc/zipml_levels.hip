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

// Column minimum and maximum (Supp. A.3): one pass over the fp32 matrix.  The rows are split
// into slabs; a thread takes V neighbouring features (one 16-byte load per row at V = 4) and the
// rows of one slab, sixteen rows requested at a time with loads that no branch can skip (rows past
// the slab repeat its last row), and stores its minima and maxima to the slab's own row of
// part[slab][2][d]; k_range_final goes through the slabs.  (An earlier version sent every
// thread's result to memory with atomics on order-preserving integer keys: 2 d slabs atomics,
// which at the 22 per ns that the memory side takes were most of its time.)
// A workgroup is TX threads across the features times 256 / TX slabs.
// A value that compares false both ways (a NaN) is never taken over, unless it is a slab's first.
constexpr int kRangeSlabsMax = 2048;
inline int64_t range_slabs_max(int64_t d)
{
    const int64_t m = ((int64_t)1 << 18) / (d > 0 ? d : 1);      // (at most 2 MiB of partial results)
    return m < 1 ? 1 : m > kRangeSlabsMax ? kRangeSlabsMax : m;
}
template <int V>
__global__ __launch_bounds__(256) void k_range_scan(const float *__restrict__ A, int64_t n,
                                                    int64_t d, int64_t lda, int64_t rows_per_slab,
                                                    int64_t nslabs, int TX, float *__restrict__ part)
{
    const int tx = threadIdx.x % TX, ty = threadIdx.x / TX;
    const int64_t j = ((int64_t)blockIdx.x * TX + tx) * V;
    const int64_t slab = (int64_t)blockIdx.y * (256 / TX) + ty;
    if (j >= d || slab >= nslabs) return;
    const int64_t i0 = slab * rows_per_slab;
    const int64_t i1 = i0 + rows_per_slab < n ? i0 + rows_per_slab : n;     // (i0 < i1: the host sized the slabs so)
    constexpr int U = V == 4 ? 16 : 8;
    float mn[V], mx[V];
    const float *col = A + j;
#pragma unroll
    for (int k = 0; k < V; ++k) mn[k] = mx[k] = col[i0 * lda + k];
    for (int64_t i = i0; i < i1; i += U) {
        float a[U][V];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float *src = col + (i + u < i1 ? i + u : i1 - 1) * lda;
            if constexpr (V == 4) {
                const float4 v = *reinterpret_cast<const float4 *>(src);
                a[u][0] = v.x; a[u][1] = v.y; a[u][2] = v.z; a[u][3] = v.w;
            } else {
                a[u][0] = *src;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < V; ++k) {
                mn[k] = a[u][k] < mn[k] ? a[u][k] : mn[k];
                mx[k] = a[u][k] > mx[k] ? a[u][k] : mx[k];
            }
    }
    float *dst = part + (size_t)slab * 2 * d + j;
#pragma unroll
    for (int k = 0; k < V; ++k) { dst[k] = mn[k]; dst[d + k] = mx[k]; }
}

// 8 features x 32 lanes that share out the slabs; lane 0 of a feature goes through the lanes' results.
__global__ __launch_bounds__(256) void k_range_final(const float *__restrict__ part, int64_t nslabs,
                                                     int64_t d, int symmetric, float *lo, float *hi)
{
    __shared__ float smn[32][8], smx[32][8];
    const int fx = threadIdx.x & 7, ly = threadIdx.x >> 3;
    const int64_t j = (int64_t)blockIdx.x * 8 + fx;
    const int64_t jc = j < d ? j : d - 1;
    const int64_t k0 = ly < nslabs ? ly : 0;
    float mn = part[(size_t)k0 * 2 * d + jc], mx = part[(size_t)k0 * 2 * d + d + jc];
    for (int64_t k = ly + 32; k < nslabs; k += 32 * 8) {
        float a[8], b[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t kk = k + 32 * u < nslabs ? k + 32 * u : k0;
            a[u] = part[(size_t)kk * 2 * d + jc];
            b[u] = part[(size_t)kk * 2 * d + d + jc];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            mn = a[u] < mn ? a[u] : mn;
            mx = b[u] > mx ? b[u] : mx;
        }
    }
    smn[ly][fx] = mn;
    smx[ly][fx] = mx;
    __syncthreads();
    if (ly != 0 || j >= d) return;
    for (int q = 1; q < 32; ++q) {
        mn = smn[q][fx] < mn ? smn[q][fx] : mn;
        mx = smx[q][fx] > mx ? smx[q][fx] : mx;
    }
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

// Per-bin moments of the normalised values; hist is [d][M][3] fp64 (count, sum t, sum t^2).
// One atomic per value and moment straight to memory ran at the rate the memory side takes
// atomics (about 22 per ns: 18-28 ms for 65,536 x 2048 values).  Here a workgroup owns F
// consecutive features -- as many as have their M bins in LDS, F a power of two up to 32 -- and
// a slab of rows, adds into LDS, and stores its bins once at the end (k_hist_merge adds the slabs).
// The counts are 32-bit integers to save LDS; the two sums are fp64: 20 bytes per bin, which is
// exactly the 160 KiB of a compute unit for 32 features x 256 bins or 8 x 1024.
//
// What the kernel is bound by is the number of cache lines in flight, not bytes or arithmetic
// (with every addition taken out it ran as long): a workgroup reads 4 F bytes of every row, the
// memory pipeline moves whole 128-byte lines, so at F = 8 three quarters of every line in flight
// are somebody else's features (and come from memory again when the workgroups that share a
// line drift apart: 1.3 to 3.9 times the matrix was fetched).  Hence the largest F that fits,
// and slabs of rows to fill the device instead of narrower blocks of features.
// A workgroup has 1024 threads: its bins leave room for one workgroup per compute unit, and its
// sixteen waves are all there is to hide the latency of the loads with.
//
// t = (a - lo) / (hi - lo) in fp64 decides the bin, floor(t M).  A division per value would be
// most of the kernel's arithmetic, so a thread keeps r = 1 / w (a correctly rounded reciprocal,
// one division per feature) and forms q = num r, then q + (num - q w) r with two fused
// operations: the classical last step of a software division, which gives the correctly rounded
// quotient from a correctly rounded reciprocal.  The bin does not rest on that: q is within 2^-51
// of the quotient either way, so q M is within 4096 * 2^-51 < 1e-11 of t M, and wherever q M comes
// closer than 1e-9 to an integer the value is divided for real.  (num == 0 gives exactly 0 both ways.)
constexpr int kHistThreads = 1024;
__device__ __forceinline__ void hist_add(float a, double l, double w, double rw, int M, double *st,
                                         double *st2, uint32_t *cf)
{
    double t = 0.0;
    int m = 0;
    if (w > 0.0) {
        const double num = (double)a - l;
        double q = num * rw;
        q = fma(fma(-q, w, num), rw, q);
        q = q < 0.0 ? 0.0 : q;
        q = q > 1.0 ? 1.0 : q;
        const double u = q * (double)M;
        int mi = (int)u;
        const double fr = u - (double)mi;
        if ((fr < 1e-9 || fr > 1.0 - 1e-9) && num != 0.0) {      // too close to an edge to trust
            q = num / w;
            q = q < 0.0 ? 0.0 : q;
            q = q > 1.0 ? 1.0 : q;
            mi = (int)(q * (double)M);
        }
        t = q;
        m = mi > M - 1 ? M - 1 : mi;
    }
    atomicAdd(cf + m, 1u);
    unsafeAtomicAdd(st + m, t);
    unsafeAtomicAdd(st2 + m, t * t);
}
// V: features per thread (4: one 16-byte load per row, when F, d, lda and the address of A allow; 1).
// out: hist itself (one slab), or the slabs' own copies [gridDim.y][d][M][3].
template <int V>
__global__ __launch_bounds__(kHistThreads) void k_hist(const float *__restrict__ A, int64_t n, int64_t d,
                                                       int64_t lda, int64_t rows_per_slab,
                                                       const float *__restrict__ lo,
                                                       const float *__restrict__ hi, int M, int F,
                                                       double *__restrict__ out)
{
    extern __shared__ __align__(16) unsigned char hist_smem[];
    double *sh = (double *)hist_smem;                        // [F][2][M] sum t, sum t^2
    uint32_t *cnt = (uint32_t *)(sh + (size_t)F * M * 2);    // [F][M] counts (a slab has fewer than 2^32 rows)
    const int tid = threadIdx.x;
    // Blocks go round the 8 dies in turn, and neighbouring blocks of features share the cache
    // lines of every row (when F < 32): block b takes features block (b % 8) * (gridDim.x / 8) +
    // b / 8, so that neighbours run on one die at about the same time.  (gridDim.x is a multiple
    // of 8; blocks past the last features block leave.)
    const int64_t fb = (int64_t)(blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8;
    const int64_t j0 = fb * F;
    if (j0 >= d) return;
    const int nf = (int)(d - j0 < F ? d - j0 : F);
    const int64_t i0 = (int64_t)blockIdx.y * rows_per_slab;
    const int64_t i1 = i0 + rows_per_slab < n ? i0 + rows_per_slab : n;
    for (int e = tid; e < nf * M * 2; e += kHistThreads) sh[e] = 0.0;
    for (int e = tid; e < nf * M; e += kHistThreads) cnt[e] = 0u;
    __syncthreads();
    // F / V threads share a row: thread t keeps the features V (t % (F / V)) ... + V - 1 for good
    // (their ranges in registers) and takes the rows t / (F / V), + 1024 / (F / V), ...  All values
    // of a round are requested before the first is used, with loads that no branch can skip (rows
    // past the slab repeat its last row and are not counted): a load behind a branch makes the
    // compiler wait for it on the spot.  Nothing in the loop reads LDS, so the additions are never
    // waited for.
    const int tpr = F / V;
    const int f = (tid % tpr) * V;
    if (i0 < i1 && f < nf) {       // (V == 4: d is a multiple of 4, so the four features live or die together)
        constexpr int U = V == 4 ? 8 : 16;
        const int rows_step = kHistThreads / tpr;
        double l[V], w[V], rw[V];
#pragma unroll
        for (int k = 0; k < V; ++k) {
            l[k] = (double)lo[j0 + f + k];
            w[k] = (double)hi[j0 + f + k] - l[k];
            rw[k] = w[k] > 0.0 ? 1.0 / w[k] : 0.0;
        }
        const float *col = A + j0 + f;
        for (int64_t i = i0 + tid / tpr; i < i1; i += (int64_t)U * rows_step) {
            float a[U][V];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t r = i + (int64_t)u * rows_step;
                const float *src = col + (r < i1 ? r : i1 - 1) * lda;
                if constexpr (V == 4) {
                    const float4 v = *reinterpret_cast<const float4 *>(src);
                    a[u][0] = v.x; a[u][1] = v.y; a[u][2] = v.z; a[u][3] = v.w;
                } else {
                    a[u][0] = *src;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i + (int64_t)u * rows_step < i1) {
#pragma unroll
                    for (int k = 0; k < V; ++k)
                        hist_add(a[u][k], l[k], w[k], rw[k], M, sh + (size_t)(f + k) * M * 2,
                                 sh + (size_t)(f + k) * M * 2 + M, cnt + (size_t)(f + k) * M);
                }
            }
        }
    }
    __syncthreads();
    double *dst = out + (size_t)blockIdx.y * ((size_t)d * M * 3) + (size_t)j0 * M * 3;
    for (int e = tid; e < nf * M * 3; e += kHistThreads) {
        const int bin = e / 3, c = e % 3, ff = bin / M, m = bin % M;
        dst[e] = c == 0 ? (double)cnt[bin] : sh[((size_t)ff * 2 + (c - 1)) * M + m];
    }
}
// hist = the slabs' copies added up in slab order
__global__ void k_hist_merge(const double *__restrict__ part, int slabs, int64_t count,
                             double *__restrict__ hist)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    double v = part[i];
    for (int k = 1; k < slabs; ++k) v += part[(size_t)k * count + i];
    hist[i] = v;
}
// Features per workgroup of k_hist (a power of two, at most 32) and its LDS bytes.
inline size_t hist_lds_bytes(int M, int F) { return (size_t)F * (size_t)M * 20; }
inline int hist_features(int M, int lds_limit)
{
    int f = 1;
    while (f < 32 && hist_lds_bytes(M, 2 * f) <= (size_t)lds_limit) f *= 2;
    return f;
}
// Room for the slabs' copies of the bin moments (beyond it, fewer slabs).
constexpr size_t kHistSlabBytes = (size_t)64 << 20;

// ---------------------------------------------------------------------------------------------
// Host dynamic program for one feature: s intervals over the M+1 bin edges m/M.
// Returns the total variance; idx[0..s] are the chosen edges.  Ties: smallest j.
// ---------------------------------------------------------------------------------------------
// The dynamic program of Sec. 3 on the device: one workgroup per feature, everything in LDS.
//   T(1, m) = V(0, m),  T(k, m) = min_{k-1 <= j <= m-1} T(k-1, j) + V(j, m),
//   V(j, m) = sum over the points in [d_j, d_m) of (d_m - t)(t - d_j), from prefix moments.
// The arithmetic is that of the host version below, operation by operation (prefix sums in index
// order, the same expression for V, the smallest j on ties), so both give the same levels.
// Thread tid takes the end points m = M - tid, M - 1023 + tid, M - 1024 - tid, ... (512 threads: the tables leave room
// for two workgroups per compute unit, and with 256 threads each the vector units idled half the time);
// in step i of the inner loop all threads of a wave read the same j, which LDS serves as a broadcast.
// LDS: 6 arrays of M+1 doubles and the argmin table (s+1) x (M+1) uint16.
__host__ __device__ inline size_t dp_lds_bytes(int M, int s)
{
    const size_t W = (size_t)M + 1;
    return 6 * W * sizeof(double) + (((size_t)s + 1) * W * sizeof(uint16_t) + 15) / 16 * 16 + 64;
}
// With sel / count (the greedy search below): the candidates of feature j are the count[j] + 1 bin
// edges sel[j][0 .. count[j]] and hist holds the moments of the intervals between them; Mcap is
// the largest number of intervals a feature can have (it sizes the tables).
constexpr int kDpThreads = 512;
__global__ __launch_bounds__(kDpThreads) void k_dp_levels(const double *__restrict__ hist,
                                                   const float *__restrict__ lo,
                                                   const float *__restrict__ hi, int64_t d, int Mgrid,
                                                   int s, float *__restrict__ levels,
                                                   uint16_t *__restrict__ grid,
                                                   double *__restrict__ objective,
                                                   const uint16_t *__restrict__ sel,
                                                   const int *__restrict__ count, int Mcap)
{
    extern __shared__ __align__(16) unsigned char dp_smem[];
    const int K = s + 1, tid = threadIdx.x, T = blockDim.x;    // (T <= kDpThreads: fewer threads for few candidates)
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
        for (int m = tid; m < W; m += T) {
            edge[m] = (double)(cand ? (int)cand[m] : m) / (double)Mgrid;
            prev[m] = INF;
        }
        __syncthreads();
        auto V = [&](int jj, int m) {
            const double dj = edge[jj], dm = edge[m];
            return -(S2[m] - S2[jj]) + (dj + dm) * (S1[m] - S1[jj]) - dj * dm * (C[m] - C[jj]);
        };
        for (int m = 1 + tid; m <= M; m += T) {
            prev[m] = V(0, m);
            arg[1 * W + m] = 0;
        }
        __syncthreads();
        for (int k = 2; k <= s; ++k) {
            // (end points in runs of T, every other run taken backwards: the work of an end point
            // grows with m, and this way every thread's end points add up to about the same)
            for (int e0 = 0; e0 < W; e0 += T) {
                const int m = M - (((e0 / T) & 1) ? e0 + T - 1 - tid : e0 + tid);   // from M down
                if (m < 0) continue;
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

// the slabs' minima and maxima of the range scan
static size_t range_bytes(int64_t d) { return (size_t)round_up(d * 8 * range_slabs_max(d), 256); }
static size_t levels_workspace_bytes(int64_t d, int n_candidates)
{
    size_t keys = range_bytes(d);
    size_t hist = (size_t)d * (size_t)n_candidates * 3 * sizeof(double);
    size_t objective = (size_t)d * sizeof(double);     // per-feature value of the dynamic program
    // candidates left by the greedy search: bin edges [d][n_candidates + 1] uint16, their number [d]
    size_t greedy = n_candidates > 0 ? (size_t)round_up(d * ((int64_t)n_candidates + 1) * 2, 256) + (size_t)d * 4 : 0;
    size_t slabs = n_candidates > 0 ? kHistSlabBytes : 0;    // the slabs' copies of the bin moments
    return (size_t)round_up((int64_t)(keys + hist + objective + greedy), 256) + slabs;
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

    if (!(flags & ZIPML_RANGE_GIVEN)) {
        // 16-byte loads when every row segment of a thread is aligned and whole
        const bool vec4 = d % 4 == 0 && lda % 4 == 0 && ((uintptr_t)A_dev & 15) == 0;
        const int64_t ncg = vec4 ? d / 4 : d;                  // threads across a row
        int TX = 256;
        while (TX > 8 && TX / 2 >= ncg) TX /= 2;
        // slabs of rows: enough threads to fill the device, at least 16 rows each
        int64_t slabs = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>((n + 15) / 16, range_slabs_max(d)),
                                                               (int64_t)262144 / ncg + 1));
        const int64_t rows_per_slab = (n + slabs - 1) / slabs;
        slabs = (n + rows_per_slab - 1) / rows_per_slab;
        float *part = (float *)workspace_dev;
        const dim3 grid((unsigned)((ncg + TX - 1) / TX), (unsigned)((slabs + 256 / TX - 1) / (256 / TX)));
        if (vec4)
            hipLaunchKernelGGL(k_range_scan<4>, grid, dim3(256), 0, s, A_dev, n, d, lda, rows_per_slab, slabs, TX, part);
        else
            hipLaunchKernelGGL(k_range_scan<1>, grid, dim3(256), 0, s, A_dev, n, d, lda, rows_per_slab, slabs, TX, part);
        hipLaunchKernelGGL(k_range_final, dim3((unsigned)((d + 7) / 8)), dim3(256), 0, s, part, slabs, d,
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
    double *hist_dev = (double *)((unsigned char *)workspace_dev + range_bytes(d));
    const int64_t hcount = d * (int64_t)M * 3;
    int lds_limit = 0, dev = 0;
    if (HIP_FAILED(hipGetDevice(&dev)) ||
        HIP_FAILED(hipDeviceGetAttribute(&lds_limit, hipDeviceAttributeMaxSharedMemoryPerBlock, dev)))
        return ZIPML_ELAUNCH;
    {
        // Blocks of F features, F the most that fit in LDS (whole cache lines at 32), times slabs
        // of rows: as many as make the rounds of workgroups come out even, and as have room for
        // their copies of the bin moments, which k_hist_merge adds up.
        int cus = 0;
        if (HIP_FAILED(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev))) return ZIPML_ELAUNCH;
        int F = hist_features(M, lds_limit);
        // development override: a power of two that fits
        if (const long long v = knob(ZIPML_KNOB_HIST_FEATURES); v >= 1 && v <= F && (v & (v - 1)) == 0) F = (int)v;
        const size_t hl = hist_lds_bytes(M, F);
        if (hl > (size_t)lds_limit) return ZIPML_EUNSUPPORTED;
        const int64_t fblocks = (d + F - 1) / F;
        const int64_t per_cu = std::min<int64_t>(2, (int64_t)lds_limit / (int64_t)hl);   // (2048 threads)
        const int64_t room = (int64_t)cus * per_cu;
        const int64_t hs_max = std::min<int64_t>(std::min<int64_t>(64, (n + 1023) / 1024),
                                                 (int64_t)(kHistSlabBytes / ((size_t)hcount * 8)));
        int64_t hs = 1;
        double best = 0.0;
        for (int64_t c = 1; c <= std::max<int64_t>(1, hs_max); ++c) {
            const double cost = (double)((fblocks * c + room - 1) / room) / (double)c + 0.002 * (double)c;
            if (c == 1 || cost < best) { best = cost; hs = c; }
        }
        const int64_t hrows = (n + hs - 1) / hs;
        hs = (n + hrows - 1) / hrows;
        if (fblocks > 0x7fffffff) return ZIPML_EINVAL;
        double *slabs_dev = (double *)((unsigned char *)workspace_dev +
                                       round_up((int64_t)(levels_workspace_bytes(d, M) - kHistSlabBytes), 256));
        // 16-byte loads when every row segment of a thread is aligned and whole
        const bool vec4 = F % 4 == 0 && d % 4 == 0 && lda % 4 == 0 && ((uintptr_t)A_dev & 15) == 0;
        auto *kern = vec4 ? k_hist<4> : k_hist<1>;
        if (HIP_FAILED(hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)hl)))
            return ZIPML_ELAUNCH;
        hipLaunchKernelGGL(kern, dim3((unsigned)round_up(fblocks, 8), (unsigned)hs), dim3(kHistThreads), hl, s, A_dev, n, d, lda,
                           hrows, lo_dev, hi_dev, M, F, hs == 1 ? hist_dev : slabs_dev);
        if (hs > 1)
            hipLaunchKernelGGL(k_hist_merge, dim3((unsigned)((hcount + 255) / 256)), dim3(256), 0, s, slabs_dev,
                               (int)hs, hcount, hist_dev);
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
        const int dp_threads = greedy ? std::min(kDpThreads, std::max(64, (int)round_up(Mcap + 1, 64))) : kDpThreads;
        hipLaunchKernelGGL(k_dp_levels, dim3(blocks), dim3(dp_threads), dp_lds, s, hist_dev, lo_dev, hi_dev, d,
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
