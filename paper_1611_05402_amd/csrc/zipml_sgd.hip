// zipml_sgd_epoch / zipml_debug_step: double-sampled minibatch SGD on packed low-bit data.
//
// Method: Sec. 2.2 eq. (5), g = mean_i Q1(a_i)(Q2(a_i)^T x - b_i); end-to-end variant of Supp. C-E.
//
// Decomposition (feature-owner): workgroup w owns a block of 32*GQ features for the whole epoch and
// keeps its slice of the model in LDS.  Per step it
//   1. takes the partial dot products of the `batch` samples over its features from copy 2
//      (sample-major units) and adds them into a device-wide accumulator (device-scope atomics),
//   2. polls the accumulator until every workgroup's contribution has arrived,
//   3. forms the residuals, takes its slice of the mean gradient from copy 1 (feature-major
//      units) and updates its slice of the model, locally.
// A step moves little data and is bound by the latency of that one device-wide exchange, so the
// kernel is organised around the exchange:
//   - one trip instead of three.  A 64-bit accumulator word carries an arrival count in its top
//     10 bits and the sum, as a biased fixed-point integer, below: one atomic add per (workgroup,
//     sample) delivers data and arrival together, so there is no "wait until my atomics are
//     done", no separate barrier and no read of the sums after it.  Integer addition is
//     associative, so the sums -- and with them the whole epoch -- do not depend on the order in
//     which the workgroups arrive.  The fixed-point scale of a step is derived from a bound on
//     the partial sums that every workgroup tracks identically (see sgd_steps);
//   - the packed data does not depend on the model.  Every thread owns the same units (sample x
//     feature group for the dot pass, feature x sample group for the gradient pass) in every
//     step and fetches them into registers ahead of time: directly behind the atomics of step t
//     it requests copy 1 of step t+1 and copy 2 of step t+2.  The loads then travel while the
//     exchange is under way (loads of a wave, and of a compute unit's memory pipeline, return in
//     order: requested before the atomics they would hold back the exchange by their own latency;
//     behind them, the poll that is queued after them returns when both are done);
//   - exchanged data moves only through device-scope atomics / loads, so no cache write-back or
//     invalidation is ever needed;
//   - workgroup barriers inside a step order LDS traffic only (lds_barrier).
// End-to-end mode adds two small exchanges per step (the l2 norms of model and gradient), each
// closed by a grid barrier (one monotonically increasing arrival counter).
// Minibatches too large for one exchange are taken in chunks, shared out over replicas of the
// workgroups (zipml_sgd_mfma.h), and very large ones by workgroups that own samples instead of
// features (zipml_sgd_rows.h); run_sgd below chooses.
#include "zipml_device.h"
#include "zipml_host.h"

#include <math.h>
#include <algorithm>
#include <mutex>
#include <stdlib.h>

namespace zipml {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr int kMaxUpt = 4;                        // units per thread and pass that fit in registers
constexpr uint32_t kSpinLimit = 1u << 22;         // default bound of a wait: a lost workgroup ends in ZIPML_ETIMEOUT

// Exchange word: [63:54] arrival count, [53:0] sum of (value + kBias) over the arrived workgroups.
// |value| < 2^44 for every contribution, so the low field never carries into the count.
constexpr int kCountShift = 54;
constexpr long long kBias = 1ll << 44;
constexpr uint64_t kPayloadMask = (1ull << kCountShift) - 1ull;
constexpr int kScaleBits = 41;                    // 2^kexp * (bound on a sum) < 2^kScaleBits

__device__ __forceinline__ uint64_t pack_int(long long q)
{
    return (1ull << kCountShift) + (uint64_t)(q + kBias);
}
// fp32 value -> fixed point with 2^-kexp resolution (exact unless |p| < 2^(24-kexp)); values
// outside the field, infinities and NaNs are clamped so that the count stays intact.
__device__ __forceinline__ uint64_t pack_fp(float p, int kexp)
{
    const double lim = (double)(kBias - 1);
    double q = ldexp((double)p, kexp);
    q = fmin(fmax(q, -lim), lim);
    return pack_int(__double2ll_rn(q));
}
__device__ __forceinline__ long long unpack_sum(uint64_t v, int W)
{
    return (long long)(v & kPayloadMask) - (long long)W * kBias;
}

enum Mode { kAffine = 0, kTable = 1, kInt = 2 };

struct SgdArgs {
    const uint32_t *p1, *p2;
    const uint32_t *p1s, *p2s;   // symmetrised estimator: copy 2 feature-major, copy 1 sample-major
    int avg;                     // 1: symmetrised estimator (matrix-core loop only)
    const float *levels;
    const uint16_t *grid;
    const float *b;
    float *x;
    int64_t nb64, n32;     // sample blocks of copy 2 (64 rows), sample groups of copy 1 (32 rows)
    int d, d32;
    int B;                 // batch
    int64_t step0;         // first step of this launch
    int nsteps;
    float lr, grid_lo, grid_step;
    float l2;              // coefficient c of the extra gradient term c * x (least-squares SVM)
    int prox;              // proximal step after the update (ZIPML_PROX_*), fp32 model only
    float prox_coef;
    int grad_bits, model_bits;
    int ident_grid;        // grid_idx[j][c] == c
    uint64_t seed;
    uint32_t epoch;
    int GQ, W;             // feature groups per workgroup, workgroups
    int lds_levels;        // the workgroup's slice of the level table fits in LDS
    int seg_first, seg_last;   // segments of a step run by this launch (0..3)
    int persistent;        // 1: segments are separated by in-kernel grid barriers
    // workspace
    int *status;
    uint32_t *sync;
    double *nrm;           // [2 kinds][2 slots][512] (+ 1024 spare)
    uint64_t *acc;         // [4][acc_words] exchange words
    int acc_words;
    const double *bound;   // at launch: [0] sum_j maxabs(L_j)|x_j|, [1] sum_j maxabs(L_j)^2,
                           // [2] max_j delta_j|x_j|, [3] max_j delta_j maxabs(L_j)
    int mfma;              // evenly spaced levels may take the matrix-core step loop
    const int *even;       // [kEvenBlocks] 1: the levels of that block of features are evenly spaced
    int chunks;            // a minibatch is chunks * B samples (matrix-core loop only)
    int R;                 // replicas of the W workgroups that share the chunks of a minibatch (divides chunks)
    uint64_t *gx;          // [2][R][W * 32 GQ] tagged words: gradient exchange between replicas
    uint32_t spin_limit;   // polls before a wait gives up (ZIPML_ETIMEOUT); the kernel still runs to its end
    float *gbuf;           // [d] gradient carried between launches (stepwise, grad_bits > 0)
    int xstore;            // 1: the matrix-core loop exchanges its sums through tagged stores
    int xrow;              // words per row of xpart / xres
    int nred;              // workgroups behind the W owners that only reduce the tagged partial sums (0: the owners do)
    int red_piece;         // exchange words per piece of theirs (8 or 4)
    int npref;             // workgroups behind those that only read the packed codes of a later chunk into the cache
    uint64_t *xpart;       // [2][W][xrow] tagged partial sums, one row per workgroup
    uint64_t *xres;        // [2][xrow] tagged sums
    // debug outputs (may be null)
    int32_t *dbg_m, *dbg_acc, *dbg_gq;
    float *dbg_r, *dbg_g;
    int dbg_production;    // 1: dbg_r / dbg_g are written by the production launch (matrix-core loop)
};

// Proximal operator of lr * R at v, coordinate-wise (Sec. 2, x <- prox_{gamma R}(x - gamma g)):
// l1 norm -> soft threshold at lr * coef; coef/2 ||x||^2 -> v / (1 + lr * coef); the constraint
// ||x||_inf <= coef -> clamp.  None of them increases |v|, so the magnitude bounds that the step
// loops track for the model stay valid.
__device__ __forceinline__ float apply_prox(float v, int kind, float lr, float coef)
{
    if (kind == ZIPML_PROX_L1) {
        const float t = lr * coef;
        return v > t ? v - t : v < -t ? v + t : 0.0f;
    }
    if (kind == ZIPML_PROX_L2SQ) return __fdiv_rn(v, 1.0f + lr * coef);
    if (kind == ZIPML_PROX_BOX) return fminf(fmaxf(v, -coef), coef);
    return v;
}

// LDS arrays of one workgroup.
struct Lds {
    float *Ls;        // level slice [CW][K]        (lds_levels only)
    uint16_t *Gs;     // grid-index slice [CW][K]   (integer mode with a non-identity grid)
    float *xs, *ys, *los, *dls, *gs;   // model slice, delta*x, lo, delta, gradient slice  [CW]
    int *ms;          // model codes [CW]
    int *tq;          // G[j][c] * m_j [CW][K]   (end-to-end production loop, at most 4-bit codes)
    float *Lp;        // level slice with rows K + 1 apart (end-to-end production loop, lds_levels only)
    float *rs;        // residuals [Rlen]
    float *zl;        // local dot products [B+4]   (single workgroup only)
    uint32_t *zp;     // per-unit partial dot products [GQ][B]  (GQ > 1 only)
    float *gpart;     // gradient partial sums [kMaxUpt * kThreads]
    double *red;      // reduction scratch [512]
    float *wsum;      // per wave: [0..kWaves) parts of sum_i r_i, [kWaves..2kWaves) parts of
                      // sum_j lo_j x_j, [2kWaves..3kWaves) parts of sum_i |r_i|
    int *isum;        // [kWaves]
    unsigned char *mf; // arrays of the matrix-core step loop
};

// Optional per-phase timing of workgroup 0 (development builds only: -DZIPML_PHASE_TIMING).
#ifdef ZIPML_PHASE_TIMING
#define ZIPML_TICK(k)                                                      \
    do {                                                                   \
        if (w == 0 && tid == 0) {                                          \
            const long long now_ = wall_clock64();                         \
            prof_[k] += now_ - last_;                                      \
            last_ = now_;                                                  \
        }                                                                  \
    } while (0)
#else
#define ZIPML_TICK(k) do { } while (0)
#endif

__device__ __forceinline__ void vm_wait_all()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's loads, stores and atomics are done
}

// Adjacent-pair tree sum of `len` (power of two) doubles in LDS; result in a[0].
__device__ __forceinline__ void lds_tree_sum(double *a, int len)
{
    for (int stride = 1; stride < len; stride <<= 1) {
        lds_barrier();
        for (int i = threadIdx.x * 2 * stride; i + stride < len; i += kThreads * 2 * stride)
            a[i] = a[i] + a[i + stride];
    }
    lds_barrier();
}

// Signed code of the row-scaled quantiser (Supp. A.3 eq. (quant2)), fp32 decisions.
__device__ __forceinline__ int qvec_code(float v, float M, int s, float u)
{
    if (!(M > 0.0f)) return 0;
    const float a = fabsf(v);
    const float t = __fdiv_rn(a, M);
    const float y = t * (float)s;
    int l = (int)floorf(y);
    if (l > s - 1) l = s - 1;
    const float frac = y - (float)l;
    const int mag = l + (u < frac ? 1 : 0);
    return v < 0.0f ? -mag : mag;
}

// One packed unit (BITS contiguous dwords) from global memory, with the widest loads that the
// unit's alignment (the largest power of two dividing 4*BITS bytes, at most 16) allows.
template <int BITS>
__device__ __forceinline__ void load_unit(const uint32_t *__restrict__ p, uint32_t (&u)[BITS])
{
    constexpr int kAlign = (BITS % 4 == 0) ? 16 : (BITS % 2 == 0) ? 8 : 4;
    const uint32_t *q = static_cast<const uint32_t *>(__builtin_assume_aligned(p, kAlign));
#pragma unroll
    for (int k = 0; k < BITS; ++k) u[k] = q[k];
}

}  // namespace zipml
#include "zipml_sgd_mfma.h"
#include "zipml_sgd_rows.h"
#include "zipml_sgd_rows_compact.h"
#include "zipml_sgd_rows_fp4.h"
namespace zipml {

// ---- inner loops over the 32 codes of a unit (v: 32 wave-uniform fp32/int32 values in LDS) ----
template <int BITS>
__device__ __forceinline__ float unit_fma_codes(const uint32_t (&u)[BITS], const float *v, float acc)
{
    // all 32 broadcast values first (8 LDS reads in flight), then four independent fma chains
    const float4 *v4 = reinterpret_cast<const float4 *>(v);
    float4 y[8];
#pragma unroll
    for (int m = 0; m < 8; ++m) y[m] = v4[m];
    float a0 = acc, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;
#pragma unroll
    for (int m = 0; m < 8; ++m) {
        a0 = fmaf((float)unit_code<BITS>(u, 4 * m + 0), y[m].x, a0);
        a1 = fmaf((float)unit_code<BITS>(u, 4 * m + 1), y[m].y, a1);
        a2 = fmaf((float)unit_code<BITS>(u, 4 * m + 2), y[m].z, a2);
        a3 = fmaf((float)unit_code<BITS>(u, 4 * m + 3), y[m].w, a3);
    }
    return (a0 + a1) + (a2 + a3);
}

// Dot pass, table levels: acc += L[feature jb+k][code_k] * x[jb+k].  L points at feature jb.
template <int BITS>
__device__ __forceinline__ float unit_dot_table(const uint32_t (&u)[BITS], const float *L,
                                                const float *x, float acc)
{
    constexpr int K = 1 << BITS;
#pragma unroll
    for (int k = 0; k < 32; ++k) acc = fmaf(L[k * K + unit_code<BITS>(u, k)], x[k], acc);
    return acc;
}

// Gradient pass, table levels: acc = fma(L[code_k], r[k], acc) for k = 0..31 in this order.
// L points at the levels of the one feature this unit belongs to.
template <int BITS>
__device__ __forceinline__ float unit_grad_table(const uint32_t (&u)[BITS], const float *L,
                                                 const float *r, float acc)
{
#pragma unroll
    for (int k = 0; k < 32; ++k) acc = fmaf(L[unit_code<BITS>(u, k)], r[k], acc);
    return acc;
}

// Gradient pass of the end-to-end mode: the sum over the unit's 32 samples of L[code_k] * r[k] in
// fp64 (every product of two fp32 numbers is exact there), so that the mean gradient rounded to
// fp32 does not depend on how the samples of a minibatch are shared out over units and threads
// (Supp. E: Q4 decides integer codes from this gradient).
template <int BITS>
__device__ __forceinline__ double unit_grad_table_f64(const uint32_t (&u)[BITS], const float *L,
                                                      const float *r)
{
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < 32; ++k) acc = fma((double)L[unit_code<BITS>(u, k)], (double)r[k], acc);
    return acc;
}

// Integer dot pass: acc += G[jb+k][code_k] * m[jb+k]; G == nullptr means the identity grid.
template <int BITS>
__device__ __forceinline__ int unit_dot_int(const uint32_t (&u)[BITS], const uint16_t *G,
                                            const int *m, int acc)
{
    constexpr int K = 1 << BITS;
    if (G) {
#pragma unroll
        for (int k = 0; k < 32; ++k) acc += (int)G[k * K + unit_code<BITS>(u, k)] * m[k];
    } else {
#pragma unroll
        for (int k = 0; k < 32; ++k) acc += (int)unit_code<BITS>(u, k) * m[k];
    }
    return acc;
}

// ---------------------------------------------------------------------------------------------
// The step loop, specialised on how a code becomes a value (MODE) and on the number of units a
// thread owns per pass (UPT).
// FAST: the production configuration (whole steps inside one persistent launch, no debug
// outputs); everything that only the stepwise / debug launches need folds away at compile time.
// ---------------------------------------------------------------------------------------------
template <int BITS, int MODE, bool FAST, int UPT>
__device__ __forceinline__ void sgd_steps(const SgdArgs &a, const Lds &L)
{
    constexpr int K = 1 << BITS;
    constexpr bool kIsInt = MODE == kInt;
    const bool persistent = FAST ? true : a.persistent != 0;
    const int seg_first = FAST ? 0 : a.seg_first;
    const int seg_last = FAST ? 3 : a.seg_last;
    int32_t *const dbg_m = FAST ? nullptr : a.dbg_m;
    int32_t *const dbg_acc = FAST ? nullptr : a.dbg_acc;
    int32_t *const dbg_gq = FAST ? nullptr : a.dbg_gq;
    float *const dbg_r = FAST ? nullptr : a.dbg_r;
    float *const dbg_g = FAST ? nullptr : a.dbg_g;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int w = blockIdx.x;
    const int W = a.W;
    const int GQ = a.GQ;
    const int CW = 32 * GQ;
    const int B = a.B;
    const int nrg = B >= 32 ? B / 32 : 1;          // sample groups of copy 1 per step
    const bool solo = W == 1;
    const bool local = solo && persistent;         // no other workgroup or launch: all stays in LDS
    const bool grid_sync = persistent && !solo;
    const int j0 = w * CW;                         // first feature of this workgroup
    const int ngroups = (a.d32 - w * GQ) < GQ ? (a.d32 - w * GQ) : GQ;   // owned feature groups
    const float *Lg = a.levels + (size_t)j0 * K;   // global view of the owned level slice
    float *const xs = L.xs, *const ys = L.ys, *const gs = L.gs, *const rs = L.rs;
    double *const red = L.red;

    // ---- the units this thread owns, the same in every step
    // dot pass:      unit k = (sample d_i[k] of the batch, owned feature group d_g[k])
    // gradient pass: unit k = (owned feature g_c, sample group g_rg[k] of the batch)
    int d_i[UPT], d_g[UPT];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        int i = tid + k * kThreads, g = 0;
        while (i >= B && g < GQ) { i -= B; ++g; }
        d_i[k] = i;
        d_g[k] = g;       // g >= ngroups: no such unit
    }
    const int nsl = kThreads / CW;                 // threads per owned feature
    const int g_c = tid % CW, g_sl = tid / CW;
    const int g_gq = g_c >> 5, g_cin = g_c & 31;
    const bool g_live = g_gq < ngroups;

    auto load_dot_units = [&](int64_t t, uint32_t (&dst)[UPT][BITS]) {
        const int64_t row0 = t * B;
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            if (d_g[k] < ngroups) {
                const int64_t row = row0 + d_i[k];
                const int64_t g = (int64_t)w * GQ + d_g[k];
                load_unit<BITS>(a.p2 + (g * a.nb64 * 64 + row) * BITS, dst[k]);
            }
        }
    };
    auto load_grad_units = [&](int64_t t, uint32_t (&dst)[UPT][BITS]) {
        const int64_t rg0 = (t * B) / 32;
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            const int rgl = g_sl + k * nsl;
            if (g_live && rgl < nrg) {
                const int64_t g = (int64_t)w * GQ + g_gq;
                load_unit<BITS>(a.p1 + ((g * a.n32 + rg0 + rgl) * 32 + g_cin) * BITS, dst[k]);
            }
        }
    };
    constexpr int kBpt = UPT;                      // samples per thread (batch <= UPT * kThreads):
                                                   // thread tid looks after samples tid + k*kThreads
    auto load_labels = [&](int64_t t, float (&dst)[kBpt]) {
#pragma unroll
        for (int k = 0; k < kBpt; ++k) {
            const int i = tid + k * kThreads;
            if (i < B) dst[k] = a.b[t * B + i];
        }
    };

    // ---- grid barrier state (one monotonically increasing arrival counter)
    uint32_t passed = 0;
    bool dead = false;
    auto arrive_and_poll = [&]() {   // lane 0 of wave 0, after the workgroup's atomics are done
        ++passed;
        add_dev(a.sync, 1u);
        const uint32_t target = passed * (uint32_t)W;
        uint32_t spins = 0;
#pragma unroll 1
        while (!dead && load_dev(a.sync) < target) {
            if (++spins > a.spin_limit) {
                store_dev(a.status, (int)ZIPML_ETIMEOUT);
                dead = true;
            }
        }
    };

    const int64_t t_end = a.step0 + a.nsteps;
#ifdef ZIPML_PHASE_TIMING
    long long prof_[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = wall_clock64();
#endif
    // Bound on the magnitude of any partial or full dot product of the current model,
    // sum_j maxabs(L_j)|x_j|: exact at launch (host-side pre-pass), then advanced every step by a
    // bound on the model's change.  Every workgroup computes it from the same numbers in the same
    // order, so all agree on the fixed-point scale without talking to each other.
    double bound_hat = a.bound[0];
    const double lambda = a.bound[1];
    int Wp = 1;
    while (Wp < W) Wp <<= 1;
    const int s_m = (1 << (a.model_bits > 0 ? a.model_bits - 1 : 1)) - 1;

    // Combine the W per-workgroup sums of squares (fixed tree) into an fp32 l2 norm.
    auto combined_norm = [&](const double *part, double own) -> float {
        if (local) return (float)sqrt(own);
        if (wave == 0)
            for (int i = lane; i < Wp; i += kWave) red[i] = i < W ? load_dev(part + i) : 0.0;
        lds_tree_sum(red, Wp);
        const float M = (float)sqrt(red[0]);
        lds_barrier();
        return M;
    };

    // ---- register-resident packed data: copy 2 of this step and the next, copy 1 of this step
    // and the next, labels of the next step
    uint32_t c2cur[UPT][BITS], c2nxt[UPT][BITS], c1cur[UPT][BITS], c1nxt[UPT][BITS];
    float bnext[kBpt], bfut[kBpt];
#pragma unroll
    for (int k = 0; k < kBpt; ++k) bnext[k] = bfut[k] = 0.0f;
    load_dot_units(a.step0, c2cur);
    if (a.step0 + 1 < t_end) load_dot_units(a.step0 + 1, c2nxt);
    load_grad_units(a.step0, c1nxt);
    load_labels(a.step0, bnext);

    for (int64_t t = a.step0; t < t_end; ++t) {
        uint64_t *const acc = a.acc + (size_t)(t & 3) * a.acc_words;
        const int k0 = B >= 32 ? 0 : (int)((t * B) % 32);  // batch offset inside its sample group

        ZIPML_TICK(7);
        lds_barrier();     // the model slice written at the end of the previous step
        ZIPML_TICK(0);
        // fixed-point scale of this step's exchange: 2^kexp * bound_hat < 2^kScaleBits
        int kexp = 0;
        if (!kIsInt && !local) {
            int e = 0;
            (void)frexp(bound_hat, &e);
            kexp = kScaleBits - e;
            kexp = kexp < -1000 ? -1000 : kexp > 1000 ? 1000 : kexp;
        }

        // ================= segment 0: ||x||_2 partial (model quantisation only) =================
        float Mx = 0.0f, sigma = 0.0f;
        double own_sq = 0.0;
        double *nx = a.nrm + (size_t)(t & 1) * 512;
        if (kIsInt && seg_first <= 0) {
            if (tid < CW) red[tid] = (double)xs[tid] * (double)xs[tid];
            lds_tree_sum(red, CW);
            own_sq = red[0];
            lds_barrier();
            if (!local && tid == 0) store_dev(nx + w, own_sq);
            if (grid_sync) {
                vm_wait_all();
                lds_barrier();
                if (wave == 0 && lane == 0) arrive_and_poll();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");   // no load moves above the poll
            }
        }
        if (seg_last < 1) continue;

        // ================= segment 1: model codes, dot pass =====================================
        if (seg_first <= 1) {
            if (kIsInt) {
                Mx = combined_norm(nx, own_sq);
                sigma = Mx > 0.0f ? __fdiv_rn(Mx, (float)s_m) : 0.0f;
                int mine = 0;
                if (tid < CW) {
                    const int j = j0 + tid;
                    if (j < a.d) {
                        const Philox4 r = philox_block(a.seed, a.epoch, (uint64_t)t, (uint32_t)j >> 2, 3u);
                        mine = qvec_code(xs[tid], Mx, s_m, u24(philox_word(r, (uint32_t)j & 3u)));
                    }
                    L.ms[tid] = mine;
                    if (dbg_m && j < a.d) dbg_m[j] = mine;
                }
                const int part = wave_sum_dpp(mine);
                if (lane == 0) L.isum[wave] = part;
                lds_barrier();   // publishes ms[] and isum[]
                if (tid == 0) {
                    int tot = 0;
                    for (int q = 0; q < kWaves; ++q) tot += L.isum[q];
                    if (local) ((int *)L.zl)[B] = tot;
                    else add_dev(acc + B, pack_int(tot));
                }
            }
            // dot pass: the partial sums of a sample over the owned feature groups are combined in
            // LDS before they are published
            float Cq = 0.0f;
            if (MODE == kAffine) {
#pragma unroll
                for (int q = 0; q < kWaves; ++q) Cq += L.wsum[kWaves + q];
            }
            auto publish = [&](int i, float pf, int pi) {
                if (local) {
                    if (kIsInt) ((int *)L.zl)[i] = pi; else L.zl[i] = pf;
                } else {
                    add_dev(acc + i, kIsInt ? pack_int(pi) : pack_fp(pf, kexp));
                }
            };
            const bool combine = ngroups > 1;
#pragma unroll
            for (int k = 0; k < UPT; ++k) {
                if (d_g[k] < ngroups) {
                    const int jb = d_g[k] * 32;
                    float pf = 0.0f;
                    int pi = 0;
                    if (MODE == kAffine) {
                        pf = unit_fma_codes<BITS>(c2cur[k], ys + jb, pf);
                    } else if (MODE == kTable) {
                        if (a.lds_levels) pf = unit_dot_table<BITS>(c2cur[k], L.Ls + jb * K, xs + jb, pf);
                        else pf = unit_dot_table<BITS>(c2cur[k], Lg + (size_t)jb * K, xs + jb, pf);
                    } else {
                        pi = unit_dot_int<BITS>(c2cur[k], a.ident_grid ? nullptr : L.Gs + jb * K,
                                                L.ms + jb, pi);
                    }
                    if (combine) L.zp[d_g[k] * B + d_i[k]] = kIsInt ? (uint32_t)pi : __float_as_uint(pf);
                    else publish(d_i[k], Cq + pf, pi);
                }
            }
            if (combine) {
                lds_barrier();
                for (int i = tid; i < B; i += kThreads) {
                    float pf = Cq;
                    int pi = 0;
                    for (int gq = 0; gq < ngroups; ++gq) {
                        const uint32_t v = L.zp[gq * B + i];
                        if (kIsInt) pi += (int)v; else pf += __uint_as_float(v);
                    }
                    publish(i, pf, pi);
                }
            }
            // The last wave of every workgroup clears its share of the exchange words of step t+2
            // (four buffers in rotation; one workgroup clearing them all made it the last to arrive
            // at every exchange).  The workgroup is past the exchange of step t-1, so every workgroup
            // has contributed to step t-1 and has therefore finished reading step t-2, the last user
            // of that buffer.  The stores have been performed before this wave leaves the step: a
            // wave's memory operations are reported complete in order, so the poll below (or the
            // explicit wait, if the wave has no samples to poll for) cannot finish before they
            // have.  The workgroup's contributions to step t+1 come after that, and nobody adds to
            // step t+2 before having seen all contributions to step t+1 -- this workgroup's among them.
            if (grid_sync && wave == kWaves - 1) {
                uint64_t *nxt = a.acc + (size_t)((t + 2) & 3) * a.acc_words;
                const int per = (B + 1 + a.W - 1) / a.W, hi = (w + 1) * per < B + 1 ? (w + 1) * per : B + 1;
                for (int i = w * per + lane; i < hi; i += kWave) store_dev(nxt + i, (uint64_t)0);
                if (!(tid < B)) vm_wait_all();
            }
            ZIPML_TICK(1);
        }
        if (seg_last < 2) continue;

        // Rotate the register sets and request what later steps need (copy 1 of step t+1, copy 2
        // of step t+2, labels of step t+1) now, right behind the atomics: the loads travel while
        // the exchange is under way.  A wave's memory operations complete in order, and the
        // compute unit's memory pipeline keeps that order too, so the poll below cannot return
        // before these loads have; issued anywhere else their latency would add to the
        // exchange's instead of hiding behind it.
#pragma unroll
        for (int k = 0; k < UPT; ++k)
#pragma unroll
            for (int q = 0; q < BITS; ++q) {
                c1cur[k][q] = c1nxt[k][q];
                c2cur[k][q] = c2nxt[k][q];
            }
        if (persistent) {
            if (t + 1 < t_end) {
                load_grad_units(t + 1, c1nxt);
                load_labels(t + 1, bfut);
            }
            if (t + 2 < t_end) load_dot_units(t + 2, c2nxt);
        }

        // ================= segment 2: residuals, gradient pass ==================================
        if (seg_first <= 2) {
            if (kIsInt && seg_first == 2) {
                // stepwise launch: recompute the scale of the model quantiser
                Mx = combined_norm(nx, 0.0);
                sigma = Mx > 0.0f ? __fdiv_rn(Mx, (float)s_m) : 0.0f;
            }
            ZIPML_TICK(3);
            // Every thread looks after the samples tid + q*kThreads: it polls their exchange words
            // until all W contributions are in, and forms the residuals from the sums and the
            // labels it holds in registers.  The loads are issued back to back (indices are
            // clamped, not branched on): each costs a full trip to the coherence point.
            if (local) lds_barrier();   // zl[] written by all waves
            float rsum = 0.0f, rabs = 0.0f;
            if (tid < B) {
                uint64_t raw[kBpt], rawm = 0;
                if (local) {
#pragma unroll
                    for (int q = 0; q < kBpt; ++q) {
                        const int i = tid + q * kThreads;
                        raw[q] = ((const uint32_t *)L.zl)[i < B ? i : B - 1];
                    }
                    if (kIsInt) rawm = (uint64_t)(uint32_t)((const int *)L.zl)[B];
                } else {
                    uint32_t spins = 0;
#pragma unroll 1
                    for (;;) {
#pragma unroll
                        for (int q = 0; q < kBpt; ++q) {
                            const int i = tid + q * kThreads;
                            raw[q] = load_dev(acc + (i < B ? i : B - 1));
                        }
                        if (kIsInt) rawm = load_dev(acc + B);
                        bool all = !kIsInt || (int)(rawm >> kCountShift) == W;
#pragma unroll
                        for (int q = 0; q < kBpt; ++q) all = all && (int)(raw[q] >> kCountShift) == W;
                        if (all || dead) break;
                        if (++spins > a.spin_limit) {
                            store_dev(a.status, (int)ZIPML_ETIMEOUT);
                            dead = true;
                        }
                    }
                }
                const double summ = !kIsInt ? 0.0
                                  : local ? (double)(int)(uint32_t)rawm : (double)unpack_sum(rawm, W);
#pragma unroll
                for (int q = 0; q < kBpt; ++q) {
                    const int i = tid + q * kThreads;
                    if (i < B) {
                        float r;
                        if (kIsInt) {
                            const int av = local ? (int)(uint32_t)raw[q] : (int)unpack_sum(raw[q], W);
                            const double z = (double)sigma * ((double)a.grid_lo * summ +
                                                              (double)a.grid_step * (double)av);
                            r = (float)z - bnext[q];
                            if (dbg_acc && w == 0) dbg_acc[i] = av;
                        } else {
                            const float z = local ? __uint_as_float((uint32_t)raw[q])
                                                  : (float)ldexp((double)unpack_sum(raw[q], W), -kexp);
                            r = z - bnext[q];
                        }
                        rs[k0 + i] = r;
                        rsum += r;
                        rabs += fabsf(r);
                        if (dbg_r && w == 0) dbg_r[i] = r;
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < kBpt; ++q) bnext[q] = bfut[q];
            if (MODE != kInt) {
                rsum = wave_sum_dpp(rsum);
                rabs = wave_sum_dpp(rabs);
                if (lane == 0) {
                    L.wsum[wave] = rsum;
                    L.wsum[2 * kWaves + wave] = rabs;
                }
            }
            lds_barrier();    // rs[], wsum[] ready
            ZIPML_TICK(4);
            if (!kIsInt && !local) {
                // |x_j| grows by at most lr * maxabs(L_j) * mean_i |r_i| in this step
                float Rabs = 0.0f;
#pragma unroll
                for (int q = 0; q < kWaves; ++q) Rabs += L.wsum[2 * kWaves + q];
                bound_hat += fabs((double)a.lr) * (lambda * ((double)Rabs / (double)B) +
                                                   fabs((double)a.l2) * bound_hat);
            }

            ZIPML_TICK(8);
            // gradient pass: one partial sum per owned unit (a chain over its 32 samples); in the
            // end-to-end mode, where Q4 turns the gradient into integer codes, the sums are fp64
            using gsum_t = typename std::conditional<kIsInt, double, float>::type;
            gsum_t *const gpart = reinterpret_cast<gsum_t *>(L.gpart);
            gsum_t part[UPT];
#pragma unroll
            for (int k = 0; k < UPT; ++k) {
                part[k] = 0;
                const int rgl = g_sl + k * nsl;
                if (g_live && rgl < nrg) {
                    const float *rr = rs + rgl * 32;
                    // (LDS and global tables in separate calls: one pointer for both would be generic)
                    if constexpr (kIsInt) {
                        if (a.lds_levels) part[k] = unit_grad_table_f64<BITS>(c1cur[k], L.Ls + g_c * K, rr);
                        else part[k] = unit_grad_table_f64<BITS>(c1cur[k], Lg + (size_t)g_c * K, rr);
                    } else if (MODE == kAffine) {
                        part[k] = unit_fma_codes<BITS>(c1cur[k], rr, 0.0f);
                    } else if (a.lds_levels) {
                        part[k] = unit_grad_table<BITS>(c1cur[k], L.Ls + g_c * K, rr, 0.0f);
                    } else {
                        part[k] = unit_grad_table<BITS>(c1cur[k], Lg + (size_t)g_c * K, rr, 0.0f);
                    }
                }
            }
            // gpart[sample group][feature]
#pragma unroll
            for (int k = 0; k < UPT; ++k) {
                const int rgl = g_sl + k * nsl;
                if (rgl < nrg) gpart[rgl * CW + g_c] = part[k];
            }
            ZIPML_TICK(9);
            lds_barrier();
            ZIPML_TICK(10);
            if (tid < CW) {
                // the unit sums are added in sample-group order
                gsum_t sacc = 0;
                for (int r0 = 0; r0 < nrg; r0 += 8) {
                    gsum_t v[8];     // eight LDS reads in flight, then added in order
#pragma unroll
                    for (int q = 0; q < 8; ++q) v[q] = gpart[(r0 + q < nrg ? r0 + q : r0) * CW + tid];
#pragma unroll
                    for (int q = 0; q < 8; ++q)
                        if (r0 + q < nrg) sacc += v[q];
                }
                float g;
                if constexpr (kIsInt) {
                    g = (j0 + tid < a.d) ? (float)(sacc / (double)B) : 0.0f;   // the mean, rounded once
                } else {
                    g = sacc;
                    if (MODE == kAffine) {
                        float Rtot = 0.0f;
#pragma unroll
                        for (int q = 0; q < kWaves; ++q) Rtot += L.wsum[q];
                        g = L.los[tid] * Rtot + L.dls[tid] * sacc;
                    }
                    g = (j0 + tid < a.d) ? __fdiv_rn(g, (float)B) : 0.0f;
                }
                gs[tid] = g;
                if (dbg_g && j0 + tid < a.d) dbg_g[j0 + tid] = g;
            }
            if (B < 32) {
                // a short batch shares its sample group with its neighbours: clear its residuals
                lds_barrier();
                for (int i = tid; i < B; i += kThreads) rs[k0 + i] = 0.0f;
            }
            if (a.grad_bits > 0) {
                double *ng = a.nrm + 1024 + (size_t)(t & 1) * 512;
                lds_barrier();
                if (tid < CW) red[tid] = (double)gs[tid] * (double)gs[tid];
                lds_tree_sum(red, CW);
                own_sq = red[0];
                lds_barrier();
                if (!local && tid == 0) store_dev(ng + w, own_sq);
                if (!persistent && tid < CW && j0 + tid < a.d) a.gbuf[j0 + tid] = gs[tid];
                if (grid_sync) {
                    vm_wait_all();
                    lds_barrier();
                    if (wave == 0 && lane == 0) arrive_and_poll();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                }
            }
        }
        ZIPML_TICK(5);
        if (seg_last < 3) continue;

        // ================= segment 3: gradient quantisation, update ==============================
        if (a.grad_bits > 0) {
            if (!persistent && seg_first == 3 && tid < CW)
                gs[tid] = (j0 + tid < a.d) ? a.gbuf[j0 + tid] : 0.0f;
            double *ng = a.nrm + 1024 + (size_t)(t & 1) * 512;
            const float Mg = combined_norm(ng, own_sq);
            const int s_g = (1 << (a.grad_bits - 1)) - 1;
            const float sg = Mg > 0.0f ? __fdiv_rn(Mg, (float)s_g) : 0.0f;
            if (tid < CW) {
                const int j = j0 + tid;
                if (j < a.d) {
                    const Philox4 r = philox_block(a.seed, a.epoch, (uint64_t)t, (uint32_t)j >> 2, 4u);
                    const int code = qvec_code(gs[tid], Mg, s_g, u24(philox_word(r, (uint32_t)j & 3u)));
                    if (dbg_gq) dbg_gq[j] = code;
                    const float gh = sg * (float)code;
                    const float stp = a.lr * gh;
                    xs[tid] = xs[tid] - stp;
                }
            }
        } else if (tid < CW) {
            const float reg = a.l2 * xs[tid];
            const float stp = a.lr * (gs[tid] + reg);
            const float v = xs[tid] - stp;
            xs[tid] = a.prox ? apply_prox(v, a.prox, a.lr, a.prox_coef) : v;
        }
        if (MODE == kAffine) {
            // the owner threads refresh y = delta * x and the per-wave parts of sum_j lo_j x_j
            float part = 0.0f;
            if (tid < CW) {
                ys[tid] = L.dls[tid] * xs[tid];
                part = L.los[tid] * xs[tid];
            }
            part = wave_sum_dpp(part);
            if (lane == 0) L.wsum[kWaves + wave] = part;
        }
        // the barrier at the top of the next step publishes xs, ys, wsum
        ZIPML_TICK(6);
    }
    lds_barrier();
#ifdef ZIPML_PHASE_TIMING
    if (w == 0 && tid == 0)
        for (int k = 0; k < 12; ++k) ((long long *)(a.nrm + 2048))[k] = prof_[k];
#endif
}

}  // namespace zipml
#include "zipml_sgd_e2e.h"
namespace zipml {

// ---------------------------------------------------------------------------------------------
// The epoch kernel: LDS carve, one-time set-up, then the step loop of the right mode.
// ---------------------------------------------------------------------------------------------
// REP: the launch has replicas of the workgroups (a.R > 1; matrix-core loop only).  A kernel of
// its own, so that the code of the replicas costs the ordinary launch no registers.
// SOLO: 0, or the one instantiation of the matrix-core loop that this kernel holds for the plain
// estimator -- 1 + (KB - 1) + 2 XM: 64 or 128 features per workgroup, exchange through atomics or
// through tagged stores.  With all its instantiations in one kernel the loop of a production launch
// spilled some 900 scalar registers into vector lanes (85 reloads inside one loop body); a kernel
// that holds one of them spills 200, and the dense 8-bit step went from 2.97 to 2.88 us.
template <int BITS, bool INT, bool FAST, int UPT, bool REP = false, int SOLO = 0>
__global__ __launch_bounds__(kThreads) void k_sgd(SgdArgs a)
{
    constexpr int K = 1 << BITS;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int w = blockIdx.x % a.W;                // feature block; blockIdx.x / a.W: replica (matrix-core loop)
    const int CW = 32 * a.GQ;
    const int B = a.B;
    const int nrg = B >= 32 ? B / 32 : 1;
    const int Rlen = nrg * 32;                     // residual slots (zero outside the batch)
    const int j0 = w * CW;
#ifdef ZIPML_PHASE_TIMING
    // where this workgroup runs: XCC id (HW_REG_XCC_ID) and the HW_ID register (SE / CU / SIMD fields)
    if (tid == 0) {
        ((long long *)(a.nrm + 2048))[16 + 2 * blockIdx.x] = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20);
        ((long long *)(a.nrm + 2048))[17 + 2 * blockIdx.x] = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);
    }
#endif

    size_t off = 0;
    auto carve = [&](size_t bytes) { void *p = smem + off; off += (bytes + 15) & ~(size_t)15; return p; };
    Lds L;
    L.Ls = (float *)carve(a.lds_levels ? (size_t)CW * K * 4 : 0);
    L.Gs = (uint16_t *)carve(INT && !a.ident_grid ? (size_t)CW * K * 2 : 0);
    L.xs = (float *)carve(CW * 4);
    L.ys = (float *)carve(CW * 4);
    L.los = (float *)carve(CW * 4);
    L.dls = (float *)carve(CW * 4);
    L.gs = (float *)carve(CW * 4);
    L.ms = (int *)carve(CW * 4);
    L.tq = (int *)carve(INT && FAST && BITS <= 4 ? (size_t)CW * K * 4 : 0);
    L.Lp = (float *)carve(INT && FAST && a.lds_levels ? (size_t)CW * (K + 1) * 4 : 0);
    L.rs = (float *)carve((size_t)Rlen * 4);
    L.zl = (float *)carve(a.W == 1 ? (size_t)(B + 4) * 4 : 0);
    L.zp = (uint32_t *)carve(a.GQ > 1 ? (size_t)a.GQ * B * 4 : 0);
    L.gpart = (float *)carve((size_t)kMaxUpt * kThreads * (INT ? 8 : 4));   // fp64 sums in the end-to-end mode
    L.red = (double *)carve(512 * 8);
    L.wsum = (float *)carve(3 * kWaves * 4);
    L.isum = (int *)carve(kWaves * 4);
    L.mf = (unsigned char *)carve(a.mfma ? mfma_lds_bytes(a.GQ, B, a.avg ? 2 : 1) : 0);

    // ---- one-time set-up: level slice, model slice
    const float *Lg = a.levels + (size_t)j0 * K;
    if (a.lds_levels)
        for (int e = tid; e < CW * K; e += kThreads) L.Ls[e] = (j0 + e / K < a.d) ? Lg[e] : 0.0f;
    if (INT && FAST && a.lds_levels)
        for (int e = tid; e < CW * K; e += kThreads)
            L.Lp[(e / K) * (K + 1) + e % K] = (j0 + e / K < a.d) ? Lg[e] : 0.0f;
    if (INT && !a.ident_grid)
        for (int e = tid; e < CW * K; e += kThreads)
            L.Gs[e] = (j0 + e / K < a.d) ? a.grid[(size_t)j0 * K + e] : (uint16_t)0;
    for (int c = tid; c < CW; c += kThreads) L.xs[c] = (j0 + c < a.d) ? a.x[j0 + c] : 0.0f;
    // Are the levels of every owned feature evenly spaced (fp64 formula, rounded once)?  Then a
    // value is lo + code * delta and the table look-up is replaced by arithmetic.
    int ok = 1;
    if (!INT) {
        for (int e = tid; e < CW * K; e += kThreads) {
            const int jj = e / K, c = e % K;
            if (j0 + jj < a.d) {
                const double lo = (double)Lg[(size_t)jj * K], wdt = (double)Lg[(size_t)jj * K + K - 1] - lo;
                ok &= (Lg[e] == (float)(lo + ((double)c * wdt) / (double)(K - 1)));
            }
        }
    }
    const bool affine = __syncthreads_and(ok) && !INT;
    // ... and of every feature of the problem (found by the preparation kernel)?  Workgroups on
    // the matrix-core loop and on the vector loop scale their contributions differently, so that
    // choice has to be the same everywhere.
    int ok_all = 1;
    if (a.mfma && tid < Workspace::kEvenBlocks) ok_all = a.even[tid];
    const bool affine_all = __syncthreads_and(ok_all) && a.mfma != 0;
    for (int c = tid; c < CW; c += kThreads) {
        const bool live = j0 + c < a.d;
        const float lo = live ? Lg[(size_t)c * K] : 0.0f, hi = live ? Lg[(size_t)c * K + K - 1] : 0.0f;
        L.los[c] = lo;
        L.dls[c] = (float)(((double)hi - (double)lo) / (double)(K - 1));
        L.ys[c] = L.dls[c] * L.xs[c];
        L.gs[c] = 0.0f;
        L.ms[c] = 0;
    }
    for (int i = tid; i < Rlen; i += kThreads) L.rs[i] = 0.0f;
    if (tid < 3 * kWaves) L.wsum[tid] = 0.0f;
    __syncthreads();
    if (affine) {
        const float part = wave_sum_dpp(tid < CW ? L.los[tid] * L.xs[tid] : 0.0f);
        if (lane == 0) L.wsum[kWaves + wave] = part;
    }

    constexpr bool kMfmaBits = BITS == 2 || BITS == 4 || BITS == 8;
    const bool on_mfma_loop = !INT && FAST && kMfmaBits && affine_all && a.mfma;
    const bool on_e2e_loop = INT && FAST && a.W > 1;
    if (((a.chunks > 1 || a.avg) && !on_mfma_loop) ||
        (FAST && a.dbg_production && !on_mfma_loop && !on_e2e_loop)) {
        // minibatches taken in chunks and the symmetrised estimator exist on the matrix-core loop
        // only; the intermediates of a production step on that loop and on the end-to-end loop
        if (blockIdx.x == 0 && tid == 0) store_dev(a.status, (int)ZIPML_EUNSUPPORTED);
        return;
    }
    if constexpr (SOLO != 0) {
        // (the host launches this kernel for the plain estimator on the matrix-core plan, without
        // replicas or debug outputs, with the workgroup width and the exchange it was built for)
        if constexpr (!INT && FAST && kMfmaBits && !REP) {
            constexpr int kKB = 1 + ((SOLO - 1) & 1), kXM = (SOLO - 1) >> 1;
            if constexpr (kXM == 1) {
                if ((int)blockIdx.x >= a.W + a.nred) {  // a workgroup that only prefetches (a.npref > 0)
                    if (affine_all && a.mfma) sgd_prefetchers<BITS>(a);
                    return;
                }
                if ((int)blockIdx.x >= a.W) {           // a workgroup that only reduces (a.nred > 0)
                    if (affine_all && a.mfma) sgd_reducers<UPT>(a, L);
                    return;
                }
            }
            if (affine_all && a.mfma) sgd_steps_mfma<BITS, UPT, kKB, 1, false, kXM>(a, L, L.mf);
            else if (affine) sgd_steps<BITS, kAffine, FAST, UPT>(a, L);
            else sgd_steps<BITS, kTable, FAST, UPT>(a, L);
        }
    } else if constexpr (REP) {
        if constexpr (!INT && FAST && kMfmaBits) {
            if (affine_all && a.mfma) {     // (anything else has been refused above: replicas imply chunks)
                if (a.avg) {
                    if constexpr (UPT <= 2) {
                        if (a.GQ <= 2) sgd_steps_mfma<BITS, UPT, 1, 2, true, 0>(a, L, L.mf);
                        else sgd_steps_mfma<BITS, UPT, 2, 2, true, 0>(a, L, L.mf);
                    }
                } else if (a.xstore) {
                    if (a.GQ <= 2) sgd_steps_mfma<BITS, UPT, 1, 1, true, 1>(a, L, L.mf);
                    else sgd_steps_mfma<BITS, UPT, 2, 1, true, 1>(a, L, L.mf);
                } else {
                    if (a.GQ <= 2) sgd_steps_mfma<BITS, UPT, 1, 1, true, 0>(a, L, L.mf);
                    else sgd_steps_mfma<BITS, UPT, 2, 1, true, 0>(a, L, L.mf);
                }
            }
        }
    } else if constexpr (!INT && FAST && kMfmaBits) {
        if (affine_all && a.mfma) {
            if (a.avg) {
                if constexpr (UPT <= 2) {      // the plan keeps the symmetrised estimator to these
                    if (a.GQ <= 2) {
                        if (a.xstore) sgd_steps_mfma<BITS, UPT, 1, 2, false, 1>(a, L, L.mf);
                        else sgd_steps_mfma<BITS, UPT, 1, 2, false, 0>(a, L, L.mf);
                    } else {
                        if (a.xstore) sgd_steps_mfma<BITS, UPT, 2, 2, false, 1>(a, L, L.mf);
                        else sgd_steps_mfma<BITS, UPT, 2, 2, false, 0>(a, L, L.mf);
                    }
                }
            } else if (a.dbg_production) {
                if (a.GQ <= 2) sgd_steps_mfma<BITS, UPT, 1, 1, false, 2>(a, L, L.mf);
                else sgd_steps_mfma<BITS, UPT, 2, 1, false, 2>(a, L, L.mf);
            } else {
                // (the plain estimator runs on the kernels that hold one instantiation each: SOLO)
                if (blockIdx.x == 0 && tid == 0) store_dev(a.status, (int)ZIPML_EUNSUPPORTED);
                return;
            }
        } else if (affine) {
            sgd_steps<BITS, kAffine, FAST, UPT>(a, L);
        } else {
            sgd_steps<BITS, kTable, FAST, UPT>(a, L);
        }
    } else {
        if constexpr (INT && FAST) {
            // (a single workgroup is launched on the other instantiation: the host sees to it, so
            // that this one holds the end-to-end loop only and its registers)
            if (a.W > 1) sgd_steps_e2e<BITS, UPT>(a, L);
        } else if (INT) {
            sgd_steps<BITS, kInt, FAST, UPT>(a, L);
        } else if (affine) {
            sgd_steps<BITS, kAffine, FAST, UPT>(a, L);
        } else {
            sgd_steps<BITS, kTable, FAST, UPT>(a, L);
        }
    }

    // ---- write the model slice back (the replicas hold identical copies: the first one does it)
    if ((FAST || a.seg_last >= 3) && blockIdx.x < a.W)
        for (int c = tid; c < CW; c += kThreads)
            if (j0 + c < a.d) a.x[j0 + c] = L.xs[c];
}

// Launch preparation: clears the barrier counter, the status word and exchange words, checks
// block by block (kEvenBlocks of them) whether the levels are evenly spaced; one more block takes
// the magnitude bounds of the dot exchange from the levels and the current model,
//   bound[0] = sum_j maxabs(L_j) |x_j|,   bound[1] = sum_j maxabs(L_j)^2,
//   bound[2] = max_j delta_j |x_j|,       bound[3] = max_j delta_j maxabs(L_j),
// (delta_j: spacing of evenly spaced levels) in fp64 with a fixed order.
// (1024 threads: a block's share of the level tables is then two loads per thread, all in flight
// together; with 256 the launch took 10 us on 2,048 x 256 levels, now 5.5.  The bounds' block reads a
// cache line per feature through one compute unit: 19 us at 16,384 features, of an epoch of 3.3 ms.)
constexpr int kPrepThreads = 1024;
__global__ __launch_bounds__(kPrepThreads) void k_sgd_prepare(int *status, uint32_t *sync, uint64_t *acc,
                                                      int words, int clear_status,
                                                      const float *__restrict__ levels,
                                                      const float *__restrict__ x, int d, int K,
                                                      double *bound, int *even,
                                                      float *dl = nullptr, float *mid = nullptr,
                                                      int nfeat = 0, float off = 0.0f,
                                                      uint64_t *slots = nullptr, int nslots = 0,
                                                      uint64_t *tagged = nullptr, int64_t ntagged = 0)
{
    __shared__ double sb[kPrepThreads], sl[kPrepThreads], sy[kPrepThreads], sm[kPrepThreads];
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) { sync[0] = 0u; if (clear_status) status[0] = 0; }
    for (int e = i; e < words; e += gridDim.x * blockDim.x) acc[e] = 0ull;
    for (int e = i; e < nslots; e += gridDim.x * blockDim.x) slots[e] = 0ull;   // norm exchange slots
    for (int64_t e = i; e < ntagged; e += gridDim.x * blockDim.x) tagged[e] = 0ull;   // tagged exchange words
    // per-feature constants of the sample-owner kernel: delta_j and lo_j + off * delta_j (zero for padding)
    if (dl)
        for (int j = i; j < nfeat; j += gridDim.x * blockDim.x) {
            float dv = 0.0f, mv = 0.0f;
            if (j < d) {
                const float lo = levels[(size_t)j * K], hi = levels[(size_t)j * K + K - 1];
                dv = (float)(((double)hi - (double)lo) / (double)(K - 1));
                mv = lo + off * dv;
            }
            dl[j] = dv;
            mid[j] = mv;
        }
    // blocks 0 .. kEvenBlocks-1: is this block's share of the level tables evenly spaced (fp64
    // formula, rounded once)?  Asked only where the answer matters (K a multiple of 4): four
    // entries per load, the loads of a thread independent of each other.
    if (even && blockIdx.x < Workspace::kEvenBlocks) {
        const int spf = K / 4;                                   // 16-byte segments per feature
        const int64_t total = (int64_t)d * spf;
        const int64_t per = (total + Workspace::kEvenBlocks - 1) / Workspace::kEvenBlocks;
        const int64_t s_end = (blockIdx.x + 1) * per < total ? (blockIdx.x + 1) * per : total;
        int ok = 1;
        for (int64_t sg = blockIdx.x * per + threadIdx.x; sg < s_end; sg += kPrepThreads) {
            const int64_t j = sg / spf;
            const int c0 = (int)(sg % spf) * 4;
            const float *row = levels + j * K;
            const double lo = (double)row[0], wdt = (double)row[K - 1] - lo;
            const float4 v = *reinterpret_cast<const float4 *>(row + c0);
            ok &= (v.x == (float)(lo + ((double)(c0 + 0) * wdt) / (double)(K - 1)));
            ok &= (v.y == (float)(lo + ((double)(c0 + 1) * wdt) / (double)(K - 1)));
            ok &= (v.z == (float)(lo + ((double)(c0 + 2) * wdt) / (double)(K - 1)));
            ok &= (v.w == (float)(lo + ((double)(c0 + 3) * wdt) / (double)(K - 1)));
        }
        ok = __syncthreads_and(ok);
        if (threadIdx.x == 0) even[blockIdx.x] = ok;
    }
    // one more block takes the magnitude bounds (the sample-owner kernel takes its scales from the data)
    if (blockIdx.x != Workspace::kEvenBlocks || !bound) return;
    double pb = 0.0, pl = 0.0, py = 0.0, pm = 0.0;
    for (int j = threadIdx.x; j < d; j += kPrepThreads) {
        const double lo = (double)levels[(size_t)j * K], hi = (double)levels[(size_t)j * K + K - 1];
        const double m = fmax(fabs(lo), fabs(hi));
        const double delta = (double)(float)((hi - lo) / (double)(K - 1));
        pb += m * fabs((double)x[j]);
        pl += m * m;
        py = fmax(py, delta * fabs((double)x[j]));
        pm = fmax(pm, delta * m);
    }
    sb[threadIdx.x] = pb;
    sl[threadIdx.x] = pl;
    sy[threadIdx.x] = py;
    sm[threadIdx.x] = pm;
    __syncthreads();
    for (int stride = kPrepThreads / 2; stride > 0; stride >>= 1) {
        if ((int)threadIdx.x < stride) {
            sb[threadIdx.x] += sb[threadIdx.x + stride];
            sl[threadIdx.x] += sl[threadIdx.x + stride];
            sy[threadIdx.x] = fmax(sy[threadIdx.x], sy[threadIdx.x + stride]);
            sm[threadIdx.x] = fmax(sm[threadIdx.x], sm[threadIdx.x + stride]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        bound[0] = sb[0];
        bound[1] = sl[0];
        bound[2] = sy[0] * 1.000001;
        bound[3] = sm[0];
    }
}

struct Plan {
    int GQ, W, lds_levels, upt;
    int mfma;          // the plan leaves room for the matrix-core step loop
    size_t shmem;
};

static int device_limits(int &cus, int &lds)
{
    int dev = 0;
    if (HIP_FAILED(hipGetDevice(&dev))) return ZIPML_ELAUNCH;
    if (HIP_FAILED(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) ||
        HIP_FAILED(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev)))
        return ZIPML_ELAUNCH;
    return ZIPML_OK;
}

// Launch of a persistent kernel, all of whose workgroups wait for each other: it is refused unless
// the whole grid can be resident at once (workgroups per compute unit, from the kernel's registers
// and LDS, times compute units).  The runtime's cooperative launch makes the same check and, on
// top, sends such launches through a queue of their own, which costs some 20 us per call (measured:
// gaps of 14 and 11 us around the kernel instead of 3 to 5) -- a fifth of a step over 65,536 samples.
// An ordinary launch is the default; ZIPML_KNOB_COOPERATIVE_LAUNCH = 1 brings the other back.  Either
// way residency also needs the device's compute units to be free of other streams' kernels; every
// device-wide wait of these kernels is bounded, so the worst case is ZIPML_ETIMEOUT, not a hang.
static int launch_resident(const void *kern, int grid, void **params, size_t shmem, hipStream_t s)
{
    if (knob(ZIPML_KNOB_COOPERATIVE_LAUNCH) == 1)
        return HIP_FAILED(hipLaunchCooperativeKernel(kern, dim3(grid), dim3(kThreads), params, (unsigned)shmem, s))
                   ? ZIPML_ELAUNCH : ZIPML_OK;
    int cus = 0, lds = 0, per_cu = 0;
    if (int rc = device_limits(cus, lds)) return rc;
    if (HIP_FAILED(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kThreads, shmem))) return ZIPML_ELAUNCH;
    if ((int64_t)per_cu * cus < grid) return ZIPML_ELAUNCH;
    return HIP_FAILED(hipLaunchKernel(kern, dim3(grid), dim3(kThreads), params, shmem, s)) ? ZIPML_ELAUNCH : ZIPML_OK;
}

static size_t up16(size_t v) { return (v + 15) & ~(size_t)15; }
// the exchange words of one chunk (sums of `pairs` code pairs, two side words) fit a row
static bool NCwords_ok(int pairs, int64_t micro, int xrow) { return (int64_t)pairs * micro + 2 <= xrow; }

// LDS needed for GQ feature groups per workgroup; 0 if it does not fit.
static size_t plan_lds(int GQ, int bits, int64_t batch, bool int_table, bool int_mode, bool solo,
                       bool mfma, int pairs, int lds_limit, int &lds_levels)
{
    const int K = 1 << bits, CW = 32 * GQ;
    const int nrg = batch >= 32 ? (int)(batch / 32) : 1;
    lds_levels = (size_t)CW * K * 4 <= 65536 ? 1 : 0;
    const size_t total = (lds_levels ? up16((size_t)CW * K * 4) : 0) +
                         (int_table ? up16((size_t)CW * K * 2) : 0) + 6 * up16((size_t)CW * 4) +
                         (int_mode && bits <= 4 ? up16((size_t)CW * K * 4) : 0) +
                         (int_mode && lds_levels ? up16((size_t)CW * (K + 1) * 4) : 0) +
                         up16((size_t)nrg * 32 * 4) +
                         (solo ? up16((size_t)(batch + 4) * 4) : 0) +
                         (GQ > 1 ? up16((size_t)GQ * batch * 4) : 0) +
                         up16((size_t)kMaxUpt * kThreads * (int_mode ? 8 : 4)) + up16(512 * 8) +
                         up16(3 * kWaves * 4) + up16(kWaves * 4) +
                         (mfma ? up16(mfma_lds_bytes(GQ, batch, pairs)) : 0);
    return total <= (size_t)lds_limit ? total : 0;
}

// Chooses how many feature groups a workgroup owns.  A step costs one device-wide exchange whose
// latency grows with the number of workgroups, so small steps want few, fat workgroups; the
// registers that hold a thread's units (at most kMaxUpt per pass) and the number of compute units
// bound the choice from both sides.
static int target_workgroups()
{
    const long long v = knob(ZIPML_KNOB_TARGET_WORKGROUPS);   // development override
    if (v >= 1 && v <= 512) return (int)v;
    return 32;
}

static int make_plan(int64_t d32, int bits, int64_t batch, bool int_table, bool fp32_model, int pairs,
                     Plan &p)
{
    int cus = 0, lds = 0;
    if (int rc = device_limits(cus, lds)) return rc;
    const int kTargetW = target_workgroups();
    int best = 0;
    for (int GQ = 1; GQ <= 8; GQ <<= 1) {
        const int64_t W = (d32 + GQ - 1) / GQ;
        if (W > cus || W > 512) continue;
        // units per thread; two code pairs take twice the registers
        if (batch * GQ > (int64_t)(pairs == 2 ? 2 : kMaxUpt) * kThreads) break;
        // end-to-end mode: its production loop holds at most two units per thread and pass; take
        // more, thinner workgroups instead where the device has them
        if (!fp32_model && best && batch * GQ > 2 * (int64_t)kThreads) break;
        // 8-bit codes: four units per thread and pass are 64 dwords of packed data a lane in the
        // matrix-core loop, more than its registers hold (it spills); twice the workgroups with two
        // units each are faster where the device has them (B=1024, d=2048: 11.3 -> 7.3 us per step)
        if (fp32_model && bits == 8 && best && batch * GQ > 2 * (int64_t)kThreads) break;
        int ll = 0;
        // the matrix-core step loop: 2/4/8-bit codes, fp32 model, whole 64-sample blocks, more
        // than one workgroup, at most 8 feature tiles of 16 (whether the levels are evenly
        // spaced is found out by the kernel)
        const bool mfma = fp32_model && (bits == 2 || bits == 4 || bits == 8) && batch % 64 == 0 &&
                          W > 1 && GQ <= 4 && knob(ZIPML_KNOB_NO_MATRIX_CORES) <= 0;
        const size_t sh = plan_lds(GQ, bits, batch, int_table, !fp32_model, W == 1, mfma, pairs, lds, ll);
        if (!sh) break;
        best = GQ;
        p.GQ = GQ; p.W = (int)W; p.lds_levels = ll; p.shmem = sh; p.mfma = mfma ? 1 : 0;
        const int64_t units = batch * GQ;
        p.upt = units <= kThreads ? 1 : units <= 2 * kThreads ? 2 : 4;
        // stop at the preferred workgroup count -- unless a single workgroup is within reach:
        // it needs no device-wide exchange at all
        const int64_t gq_solo = d32 <= 8 ? (d32 <= 1 ? 1 : d32 <= 2 ? 2 : d32 <= 4 ? 4 : 8) : 0;
        const bool solo_possible = gq_solo && batch * gq_solo <= (int64_t)kMaxUpt * kThreads;
        if (W <= kTargetW && !(solo_possible && W > 1)) break;
    }
    return best ? ZIPML_OK : ZIPML_EUNSUPPORTED;   // batch too large for one step in registers
}

template <int BITS, bool INT>
static int launch_sgd(hipStream_t s, SgdArgs &a, const Plan &p, bool stepwise)
{
    const bool debug = a.dbg_m || a.dbg_acc || a.dbg_gq || a.dbg_r || a.dbg_g;
    // production instantiation: whole steps in one persistent launch (a single workgroup in the
    // end-to-end mode runs the general loop, which keeps everything in LDS)
    // (the end-to-end loop exists for one or two units per thread and pass: with four its
    // registers do not fit, and the plan prefers twice the workgroups anyway; larger minibatches
    // run the general loop)
    const bool fast = !stepwise && (!debug || a.dbg_production) && !(INT && (a.W == 1 || p.upt > 2));
    if (a.dbg_production && !fast) return ZIPML_EUNSUPPORTED;
    const void *kern = (const void *)k_sgd<BITS, INT, false, kMaxUpt>;
    if (fast) {
        if constexpr (INT) {
            kern = p.upt == 1 ? (const void *)k_sgd<BITS, true, true, 1> : (const void *)k_sgd<BITS, true, true, 2>;
        } else {
            kern = p.upt == 1 ? (const void *)k_sgd<BITS, false, true, 1>
                 : p.upt == 2 ? (const void *)k_sgd<BITS, false, true, 2>
                              : (const void *)k_sgd<BITS, false, true, 4>;
        }
        if constexpr (!INT && (BITS == 2 || BITS == 4 || BITS == 8)) {
            if (a.R > 1)
                kern = p.upt == 1 ? (const void *)k_sgd<BITS, false, true, 1, true>
                     : p.upt == 2 ? (const void *)k_sgd<BITS, false, true, 2, true>
                                  : (const void *)k_sgd<BITS, false, true, 4, true>;
            else if (a.mfma && !a.avg && !a.dbg_production) {
                // the plain estimator: the kernel that holds just its instantiation of the loop
                const int solo = 1 + (a.GQ <= 2 ? 0 : 1) + 2 * (a.xstore ? 1 : 0);
#define ZIPML_SOLO(U) (solo == 1 ? (const void *)k_sgd<BITS, false, true, U, false, 1> \
                     : solo == 2 ? (const void *)k_sgd<BITS, false, true, U, false, 2> \
                     : solo == 3 ? (const void *)k_sgd<BITS, false, true, U, false, 3> \
                                 : (const void *)k_sgd<BITS, false, true, U, false, 4>)
                kern = p.upt == 1 ? ZIPML_SOLO(1) : p.upt == 2 ? ZIPML_SOLO(2) : ZIPML_SOLO(4);
#undef ZIPML_SOLO
                // idle compute units take the reducing of the tagged partial sums (sgd_reducers), where
                // the loop really exchanges that way (all eight waves at work, as the kernel decides too)
                int cus = 0, lds = 0;
                if (int rc = device_limits(cus, lds)) return rc;
                const bool all_waves = !(p.upt == 1 && a.B <= 256 && a.GQ <= 2);
                const int npieces = ((int)a.B + 2 + 7) / 8;
                if (a.xstore && all_waves && cus - a.W >= npieces) {
                    // (a reducer per piece of eight words, or none: with fewer, a reducer takes its pieces
                    // one after the other, and the owners do better themselves -- tomography shape,
                    // us per step: none 6.57, 16 reducers 10.1, 32: 7.6, 64: 6.41, 65 = one per piece: 6.39;
                    // pieces of four words on twice the reducers: 6.8)
                    a.red_piece = 8;
                    a.nred = npieces;
                    // development override: 0 = none, n = that many (4 words per piece from 100 on: n - 100 of them)
                    if (const long long v = knob(ZIPML_KNOB_REDUCER_WORKGROUPS); v >= 0) {
                        a.red_piece = v >= 100 ? 4 : 8;
                        a.nred = (int)std::min<long long>(v >= 100 ? v - 100 : v, cus - a.W);
                    }
                    // what is idle even then reads ahead (sgd_prefetchers); 16-byte reads of whole segments
                    const int idle = cus - a.W - a.nred;
                    if (a.nred > 0 && idle >= 16 && ((int64_t)a.B * BITS * 4) % 16 == 0) a.npref = std::min(idle, 64);
                    if (const long long v = knob(ZIPML_KNOB_PREFETCH_WORKGROUPS); v >= 0) a.npref = a.nred > 0 ? (int)std::min<long long>(v, idle) : 0;
                }
            }
        }
    }
    if (a.R > 1 && !(fast && !INT && (BITS == 2 || BITS == 4 || BITS == 8))) return ZIPML_EUNSUPPORTED;
    if (HIP_FAILED(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)p.shmem)))
        return ZIPML_ELAUNCH;
    // exchange buffers of every replica, and the gradient exchange words behind them
    const int words = a.R * Workspace::kAccBuffers * a.acc_words + (a.R > 1 ? 2 * (int)Workspace::kGradWords : 0);
    const int K = 1 << BITS;
    double *bound = const_cast<double *>(a.bound);
    hipLaunchKernelGGL(k_sgd_prepare, dim3(Workspace::kEvenBlocks + 1), dim3(kPrepThreads), 0, s, a.status, a.sync,
                       a.acc, words, 1, a.levels, a.x, a.d, K, bound,
                       a.mfma ? const_cast<int *>(a.even) : nullptr, (float *)nullptr, (float *)nullptr, 0, 0.0f,
                       INT && !stepwise ? reinterpret_cast<uint64_t *>(a.nrm) : (uint64_t *)nullptr,
                       INT && !stepwise ? 8 * kNormSlots : 0,
                       a.xstore ? a.xpart : (uint64_t *)nullptr,
                       a.xstore ? (int64_t)a.R * 2 * (a.W + 1) * a.xrow : (int64_t)0);
    if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    if (!stepwise) {
        a.persistent = 1;
        a.seg_first = 0;
        a.seg_last = 3;
        void *params[] = {&a};
        return launch_resident(kern, a.W * a.R + a.nred + a.npref, params, p.shmem, s);
    }
    // stepwise: every segment of every step is its own launch; kernel boundaries replace barriers
    const int64_t first = a.step0, count = a.nsteps;
    a.persistent = 0;
    a.nsteps = 1;
    for (int64_t t = first; t < first + count; ++t) {
        a.step0 = t;
        // the exchange buffer that step t uses was last used by step t-4: clear it; the magnitude
        // bounds are taken from the model as it stands before this step
        uint64_t *acct = a.acc + (size_t)(t & 3) * a.acc_words;
        hipLaunchKernelGGL(k_sgd_prepare, dim3(Workspace::kEvenBlocks + 1), dim3(kPrepThreads), 0, s, a.status,
                           a.sync, acct, a.acc_words, 0, a.levels, a.x, a.d, K, bound, nullptr);
        for (int seg = 0; seg <= 3; ++seg) {
            if (seg == 0 && a.model_bits == 0) continue;
            if (seg == 3 && a.grad_bits == 0) continue;
            a.seg_first = seg;
            a.seg_last = seg;
            if (seg == 2 && a.grad_bits == 0) a.seg_last = 3;
            void *params[] = {&a};
            if (HIP_FAILED(hipLaunchKernel(kern, dim3(a.W), dim3(kThreads), params, p.shmem, s)))
                return ZIPML_ELAUNCH;
        }
    }
    return ZIPML_OK;
}

template <int BITS>
static int launch_sgd_mode(hipStream_t s, SgdArgs &a, const Plan &p, bool stepwise)
{
    return a.model_bits > 0 ? launch_sgd<BITS, true>(s, a, p, stepwise)
                            : launch_sgd<BITS, false>(s, a, p, stepwise);
}

// Sample-owner kernel for very large minibatches (zipml_sgd_rows.h).
template <int BITS>
static int launch_rows(hipStream_t s, RowsArgs &r, const float *levels, int wgs, int *even, uint64_t *acc)
{
    const int K = 1 << BITS;
    const int nfeat = r.NKB * 64;
    const size_t shmem = rows_lds_bytes(r.NKB);
    // blocks per wave and item: as many as the registers hold, fewer for narrow problems
    // (measured: short items are best at 4 and 8 bits, 5.8-5.9 TB/s; 2-bit codes want two blocks)
    int kpi = BITS == 2 ? 2 : 1;
    if (const long long v = knob(ZIPML_KNOB_ROWS_ITEM_BLOCKS); v >= 1 && v <= 32 / BITS) kpi = (int)v;   // development override
    while (kpi > 1 && (r.NKB < kWaves * kpi || (kpi & (kpi - 1)))) --kpi;
    const void *kern = nullptr;
    if constexpr (BITS == 8) kern = kpi >= 2 ? (const void *)k_sgd_rows<8, 2> : (const void *)k_sgd_rows<8, 1>;
    if constexpr (BITS == 4)
        kern = kpi >= 4 ? (const void *)k_sgd_rows<4, 4> : kpi == 2 ? (const void *)k_sgd_rows<4, 2>
                                                                   : (const void *)k_sgd_rows<4, 1>;
    if constexpr (BITS == 2)
        kern = kpi >= 4 ? (const void *)k_sgd_rows<2, 4> : kpi == 2 ? (const void *)k_sgd_rows<2, 2>
                                                                   : (const void *)k_sgd_rows<2, 1>;
    if (r.p1s) {     // symmetrised estimator: the default item sizes only
        kpi = BITS == 2 && r.NKB >= 2 * kWaves ? 2 : 1;
        if constexpr (BITS == 8) kern = (const void *)k_sgd_rows<8, 1, true>;
        if constexpr (BITS == 4) kern = (const void *)k_sgd_rows<4, 1, true>;
        if constexpr (BITS == 2) kern = kpi == 2 ? (const void *)k_sgd_rows<2, 2, true> : (const void *)k_sgd_rows<2, 1, true>;
    }
    size_t lds_bytes = shmem;
    if constexpr (BITS == 2) {
        // 2-bit codes, plain estimator: the dot pass on the 4-bit floating-point matrix instruction
        // (zipml_sgd_rows_fp4.h) where its digits fit in LDS; an explicit item size keeps the
        // integer kernel (development, A/B)
        int cus = 0, lds = 0;
        if (int rc = device_limits(cus, lds)) return rc;
        const long long item_knob = knob(ZIPML_KNOB_ROWS_ITEM_BLOCKS);
        const int tm_forced = item_knob == 101 || item_knob == 102 ? (int)item_knob - 100 : 0;   // development, tests
        if (!r.p1s && (item_knob < 1 || tm_forced)) {
            // the larger tile (128 or 64 samples) that divides the minibatch, leaves every workgroup
            // at least two tiles and fits in LDS
            for (int tm = 2; tm >= 1; tm >>= 1) {
                if (tm_forced && tm != tm_forced) continue;
                if (r.B % (64 * tm) != 0 || (!tm_forced && tm > 1 && r.B / (64 * tm) < 2 * (int64_t)wgs)) continue;
                if (rows_fp4_lds_bytes(r.NKB, tm) > (size_t)lds) continue;
                kern = tm == 2 ? (const void *)k_sgd_rows_fp4<2> : (const void *)k_sgd_rows_fp4<1>;
                lds_bytes = rows_fp4_lds_bytes(r.NKB, tm);
                break;
            }
        }
    }
    if (HIP_FAILED(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes)))
        return ZIPML_ELAUNCH;
    // status word, barrier counter, evenly-spaced check (no exchange words to clear)
    hipLaunchKernelGGL(k_sgd_prepare, dim3(Workspace::kEvenBlocks + 1), dim3(kPrepThreads), 0, s, r.status, r.sync,
                       acc, 0, 1, levels, r.x, r.d, K, (double *)nullptr, even, const_cast<float *>(r.dl),
                       const_cast<float *>(r.mid), nfeat, BITS == 8 ? 128.0f : 0.0f);
    if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    void *params[] = {&r};
    return launch_resident(kern, wgs, params, lds_bytes, s);
}

static int run_sgd(void *stream, const void *packed1_dev, const void *packed2_dev,
                   const void *packed1s_dev, const void *packed2s_dev, const float *levels_dev, const uint16_t *grid_idx_dev, float grid_lo,
                   float grid_step, int grid_max, const float *b_dev, int64_t n, int64_t d, int bits,
                   float *x_dev, int64_t batch, float lr, float l2, int grad_bits, int model_bits,
                   uint64_t seed, uint32_t epoch, int flags, int64_t step0, int64_t nsteps,
                   int32_t *dbg_m, int32_t *dbg_acc, float *dbg_r, float *dbg_g, int32_t *dbg_gq,
                   void *workspace_dev, size_t workspace_bytes, int prox = ZIPML_PROX_NONE,
                   float prox_coef = 0.0f, int *status_dev = nullptr)
{
    if (!packed1_dev || !packed2_dev || !levels_dev || !b_dev || !x_dev) return ZIPML_EINVAL;
    if (prox != ZIPML_PROX_NONE && prox != ZIPML_PROX_L1 && prox != ZIPML_PROX_L2SQ && prox != ZIPML_PROX_BOX)
        return ZIPML_EINVAL;
    if (prox != ZIPML_PROX_NONE && !(prox_coef >= 0.0f)) return ZIPML_EINVAL;
    if (prox != ZIPML_PROX_NONE && model_bits > 0) return ZIPML_EUNSUPPORTED;   // fp32 model only
    if (n <= 0 || d <= 0 || !valid_bits(bits) || batch <= 0 || n % batch != 0) return ZIPML_EINVAL;
    if (!(batch == 4 || batch == 8 || batch == 16 || batch % 32 == 0)) return ZIPML_EINVAL;
    if (n > (int64_t)1 << 40 || d > (1 << 24)) return ZIPML_EINVAL;
    if (model_bits != 0 && (model_bits < 2 || model_bits > 8)) return ZIPML_EINVAL;
    if (grad_bits != 0 && (grad_bits < 2 || grad_bits > 8)) return ZIPML_EINVAL;
    if (epoch >= (1u << 24)) return ZIPML_EINVAL;
    if (step0 < 0 || nsteps < 0 || step0 + nsteps > n / batch) return ZIPML_EINVAL;
    if (flags & ~(ZIPML_SGD_STEPWISE | ZIPML_SGD_AVERAGED | ZIPML_SGD_PRODUCTION)) return ZIPML_EINVAL;
    if (flags & ZIPML_SGD_AVERAGED) return ZIPML_EUNSUPPORTED;
    const bool production = (flags & ZIPML_SGD_PRODUCTION) != 0;
    if (production) {
        // the intermediates of the production launch: residuals and gradient of an fp32-model
        // step (matrix-core loop), all five outputs of an end-to-end step
        if (flags & ZIPML_SGD_STEPWISE) return ZIPML_EINVAL;
        if (!(dbg_r || dbg_g || dbg_m || dbg_acc || dbg_gq)) return ZIPML_EINVAL;
        if (model_bits == 0 && (dbg_m || dbg_acc || dbg_gq)) return ZIPML_EINVAL;
        if (packed1s_dev || packed2s_dev) return ZIPML_EUNSUPPORTED;
    }
    if (grad_bits > 0 && model_bits == 0) return ZIPML_EUNSUPPORTED;
    if (!(l2 >= 0.0f)) return ZIPML_EINVAL;
    if (l2 != 0.0f && model_bits > 0) return ZIPML_EUNSUPPORTED;   // the c*x term is not quantised here
    const bool avg = packed1s_dev != nullptr || packed2s_dev != nullptr;
    if (avg) {
        // symmetrised estimator: both extra arrays, fp32 model, production launch, matrix-core loop
        if (!packed1s_dev || !packed2s_dev) return ZIPML_EINVAL;
        if (!aligned16(packed1s_dev) || !aligned16(packed2s_dev)) return ZIPML_EALIGN;
        if (model_bits > 0 || (flags & ZIPML_SGD_STEPWISE) || dbg_m || dbg_acc || dbg_r || dbg_g || dbg_gq ||
            !(bits == 2 || bits == 4 || bits == 8) || batch % 64 != 0)
            return ZIPML_EUNSUPPORTED;
    }
    if (model_bits > 0) {
        if (!grid_idx_dev || grid_max < (1 << bits) - 1 || grid_max > 65535) return ZIPML_EINVAL;
        const int64_t s_m = ((int64_t)1 << (model_bits - 1)) - 1;
        if ((int64_t)grid_max * s_m * round_up(d, 32) >= ((int64_t)1 << 31)) return ZIPML_ERANGE;
    }
    if (!aligned16(packed1_dev) || !aligned16(packed2_dev) || !aligned16(levels_dev) ||
        !aligned16(b_dev) || !aligned16(x_dev) || !aligned16(workspace_dev) ||
        (grid_idx_dev && !aligned16(grid_idx_dev)))
        return ZIPML_EALIGN;
    if (!workspace_dev || workspace_bytes < zipml_workspace_bytes(n, d, bits, batch, 0))
        return ZIPML_EWORKSPACE;
    if (nsteps == 0) return ZIPML_OK;

    hipStream_t s = entry_stream(stream);
    const Layout lay = make_layout(n, d, bits);
    const bool ident = model_bits > 0 && grid_max == (1 << bits) - 1;
    Plan p{};
    int64_t chunks = 1, micro = batch;
    const int pairs = avg ? 2 : 1;
    int rc = make_plan(lay.d32, bits, batch, model_bits > 0 && !ident, model_bits == 0, pairs, p);
    const bool stepwise = (flags & ZIPML_SGD_STEPWISE) != 0;
    const bool debug = dbg_m || dbg_acc || dbg_r || dbg_g || dbg_gq;
    int replicas = 1;
    int64_t forced = 0;
    if (knob(ZIPML_KNOB_CHUNK_SAMPLES) > 0) forced = knob(ZIPML_KNOB_CHUNK_SAMPLES);   // development override: chunk size
    if (production && (rc != ZIPML_OK || (model_bits == 0 && !p.mfma) || (model_bits > 0 && p.W == 1)))
        return ZIPML_EUNSUPPORTED;
    const bool split_ok = model_bits == 0 && !stepwise && !debug && batch % 64 == 0 &&
                          (bits == 2 || bits == 4 || bits == 8);
    if (split_ok && (rc == ZIPML_EUNSUPPORTED || (rc == ZIPML_OK && p.mfma && forced > 0 && forced < batch))) {
        // A minibatch too large for one exchange is taken in equal chunks (matrix-core loop only:
        // the kernel reports ZIPML_EUNSUPPORTED through the status word if the levels turn out
        // not to be evenly spaced).  The largest chunk whose plan reaches the preferred number of
        // workgroups is taken (fewer, fatter workgroups leave more compute units for replicas),
        // else the largest that fits at all.
        int cus = 0, lds = 0;
        if (int lrc = device_limits(cus, lds)) return lrc;
        const int64_t w_goal = std::max<int64_t>(target_workgroups(), (lay.d32 + 3) / 4);
        bool have = false;
        for (int64_t c = 2; c <= batch / 64; ++c) {
            if (batch % c != 0 || (batch / c) % 64 != 0) continue;
            if (forced > 0 && batch / c != forced) continue;
            Plan q{};
            if (make_plan(lay.d32, bits, batch / c, false, true, pairs, q) != ZIPML_OK || !q.mfma) continue;
            if (!have || q.W <= w_goal) {
                p = q;
                chunks = c;
                micro = batch / c;
                rc = ZIPML_OK;
                have = true;
            }
            if (q.W <= w_goal) break;
        }
        if (have) {
            // The chunks of a minibatch are independent: R replicas of the W workgroups take every
            // R-th chunk each (R a power of two that divides the number of chunks).
            int64_t cap = std::min<int64_t>(cus / p.W, Workspace::kMaxReplicas);
            if (const long long v = knob(ZIPML_KNOB_MAX_REPLICAS); v >= 1) cap = std::min<int64_t>(cap, v);   // development override
            while (replicas * 2 <= cap && chunks % (replicas * 2) == 0) replicas *= 2;
        }
    }
    // Very large minibatches: workgroups that own samples instead of features need no exchange
    // per sample (evenly spaced levels only: the kernel reports ZIPML_EUNSUPPORTED through the
    // status word otherwise, as for chunked minibatches).
    {
        // It pays from about two tiles of 64 samples per compute unit on (a step costs two
        // device-wide barriers and a reduction over all workgroups), earlier for wide problems.
        int64_t rows_min = lay.d_pad >= 8192 ? Workspace::kRowsMinBatch : 2 * Workspace::kRowsMinBatch;
        // development override (not below the workspace's rule)
        if (const long long v = knob(ZIPML_KNOB_ROWS_MIN_BATCH); v >= Workspace::kRowsMinBatch) rows_min = v;
        int cus = 0, lds = 0;
        if (int lrc = device_limits(cus, lds)) return lrc;
        const int NKB = (int)((lay.d32 + 1) / 2);
        // (the kernel's per-lane byte offsets are 32 bits wide: one feature group of copy 2 must fit)
        if (split_ok && batch >= rows_min && batch / 64 >= cus &&
            rows_lds_bytes(NKB) <= (size_t)lds && lay.n_pad * bits * 4 < ((int64_t)1 << 32) &&
            knob(ZIPML_KNOB_NO_MATRIX_CORES) <= 0) {
            unsigned char *wsb = (unsigned char *)workspace_dev;
            float *rows = (float *)(wsb + Workspace::sgd_bytes(batch) + (size_t)round_up(d, 64) * 4);
            int wgs = std::min(cus, Workspace::kMaxRowsWgs);
            if (const long long v = knob(ZIPML_KNOB_ROWS_WORKGROUPS); v >= 1 && v <= Workspace::kMaxRowsWgs) wgs = (int)v;   // development override
            RowsArgs r{};
            r.p1 = (const uint32_t *)packed1_dev;
            r.p2 = (const uint32_t *)packed2_dev;
            r.p1s = avg ? (const uint32_t *)packed1s_dev : nullptr;
            r.p2s = avg ? (const uint32_t *)packed2s_dev : nullptr;
            r.b = b_dev;
            r.x = x_dev;
            r.dl = rows;
            r.mid = rows + (size_t)NKB * 64;
            r.part = rows + (size_t)2 * NKB * 64;
            r.n_pad = lay.n_pad;
            r.n32 = lay.n32;
            r.d = (int)d;
            r.d32 = (int)lay.d32;
            r.NKB = NKB;
            r.B = batch;
            r.step0 = step0;
            r.nsteps = (int)nsteps;
            r.lr = lr;
            r.l2 = l2;
            r.prox = prox;
            r.prox_coef = prox_coef;
            r.status = status_dev ? status_dev : (int *)(wsb + Workspace::kStatus);
            r.sync = (uint32_t *)(wsb + Workspace::kSync);
            r.even = (const int *)(wsb + Workspace::kEven);
            r.spin_limit = kSpinLimit;
            // test hook: make every wait give up early
            if (const long long v = knob(ZIPML_KNOB_SPIN_LIMIT); v >= 0 && v <= (long long)kSpinLimit) r.spin_limit = (uint32_t)v;
            int *even = (int *)(wsb + Workspace::kEven);
            uint64_t *acc = (uint64_t *)(wsb + Workspace::kAcc);
            switch (bits) {
                case 2: return launch_rows<2>(s, r, levels_dev, wgs, even, acc);
                case 4: return launch_rows<4>(s, r, levels_dev, wgs, even, acc);
                case 8: return launch_rows<8>(s, r, levels_dev, wgs, even, acc);
            }
        }
    }
    if (rc) return rc;
    if (avg && !p.mfma) return ZIPML_EUNSUPPORTED;   // e.g. a problem that fits one workgroup

    unsigned char *ws = (unsigned char *)workspace_dev;
    SgdArgs a{};
    a.p1 = (const uint32_t *)packed1_dev;
    a.p2 = (const uint32_t *)packed2_dev;
    a.p1s = (const uint32_t *)packed1s_dev;
    a.p2s = (const uint32_t *)packed2s_dev;
    a.avg = avg ? 1 : 0;
    a.levels = levels_dev;
    a.grid = grid_idx_dev;
    a.b = b_dev;
    a.x = x_dev;
    a.nb64 = lay.nb64;
    a.n32 = lay.n32;
    a.d = (int)d;
    a.d32 = (int)lay.d32;
    a.B = (int)micro;
    a.chunks = (int)chunks;
    a.R = replicas;
    a.step0 = step0;
    a.nsteps = (int)nsteps;
    a.lr = lr;
    a.l2 = l2;
    a.prox = prox;
    a.prox_coef = prox_coef;
    a.grid_lo = grid_lo;
    a.grid_step = grid_step;
    a.grad_bits = grad_bits;
    a.model_bits = model_bits;
    a.ident_grid = ident ? 1 : 0;
    a.seed = seed;
    a.epoch = epoch;
    a.GQ = p.GQ;
    a.W = p.W;
    a.lds_levels = p.lds_levels;
    a.mfma = (p.mfma && !stepwise && (!debug || production)) ? 1 : 0;   // the matrix-core loop exists in the production launch only
    a.dbg_production = production ? 1 : 0;
    a.spin_limit = kSpinLimit;
    // test hook: make every wait give up early
    if (const long long v = knob(ZIPML_KNOB_SPIN_LIMIT); v >= 0 && v <= (long long)kSpinLimit) a.spin_limit = (uint32_t)v;
    a.status = status_dev ? status_dev : (int *)(ws + Workspace::kStatus);
    a.sync = (uint32_t *)(ws + Workspace::kSync);
    a.nrm = (double *)(ws + Workspace::kNorm);
    a.acc = (uint64_t *)(ws + Workspace::kAcc);
    a.bound = (const double *)(ws + Workspace::kBound);
    a.even = (const int *)(ws + Workspace::kEven);
    a.acc_words = (int)Workspace::acc_words(micro);
    a.gx = a.acc + (size_t)replicas * Workspace::kAccBuffers * a.acc_words;
    // the exchange buffers of all replicas and the gradient exchange words must fit what
    // zipml_workspace_bytes provides for this batch (they do by construction: checked anyway)
    {
        const size_t used = ((size_t)replicas * Workspace::kAccBuffers * a.acc_words +
                             (replicas > 1 ? 2 * Workspace::kGradWords : 0)) * 8;
        if (Workspace::kAcc + used > Workspace::sgd_bytes(batch) ||
            (replicas > 1 && (size_t)replicas * p.W * 32 * p.GQ > Workspace::kGradWords))
            return ZIPML_EWORKSPACE;
    }
    a.gbuf = (float *)(ws + Workspace::sgd_bytes(batch));
    // Exchange through tagged stores: the matrix-core loop with all eight waves at work and enough
    // (workgroups x samples) for the atomics to be what a step waits for.  Replicas have rows and
    // results of their own (the plain estimator only), sized for their chunk, where the room that
    // zipml_workspace_bytes provides for one launch of this minibatch holds them all.
    {
        // (by itself: from 128 workgroups and 32,768 workgroups x samples on.  What the atomics cost
        // grows with the workgroups that add to one word: at the same 65,536 atomics per step 128
        // workgroups x 512 samples take 9.1 us per step with atomics and 6.0 with tagged stores, 64 x
        // 1,024 take 4.8 and 5.7.)
        long long xmin = knob(ZIPML_KNOB_STORE_EXCHANGE_MIN);
        const bool automatic = xmin < 0;
        if (automatic) xmin = 32768;
        const bool all_waves = !(p.upt == 1 && micro <= 256 && p.GQ <= 2);
        a.xstore = (a.mfma && (replicas == 1 || !avg) && all_waves && p.W > 1 && !production &&
                    (long long)p.W * micro >= xmin && (!automatic || p.W >= 128)) ? 1 : 0;
        a.xrow = (int)Workspace::xchg_row_words(replicas > 1 ? micro : batch);
        a.xpart = (uint64_t *)(ws + Workspace::xchg_offset(d, batch));
        a.xres = a.xpart + (size_t)2 * p.W * a.xrow;
        if (a.xstore && (p.W > 256 || NCwords_ok(avg ? 2 : 1, micro, a.xrow) == false)) a.xstore = 0;
        if (a.xstore && (size_t)replicas * 2 * (p.W + 1) * a.xrow * 8 > Workspace::xchg_bytes(d, batch)) a.xstore = 0;
    }
    a.dbg_m = dbg_m; a.dbg_acc = dbg_acc; a.dbg_r = dbg_r; a.dbg_g = dbg_g; a.dbg_gq = dbg_gq;
    switch (bits) {
        case 1: return launch_sgd_mode<1>(s, a, p, stepwise);
        case 2: return launch_sgd_mode<2>(s, a, p, stepwise);
        case 3: return launch_sgd_mode<3>(s, a, p, stepwise);
        case 4: return launch_sgd_mode<4>(s, a, p, stepwise);
        case 5: return launch_sgd_mode<5>(s, a, p, stepwise);
        case 6: return launch_sgd_mode<6>(s, a, p, stepwise);
        case 7: return launch_sgd_mode<7>(s, a, p, stepwise);
        case 8: return launch_sgd_mode<8>(s, a, p, stepwise);
    }
    return ZIPML_EINVAL;
}

}  // namespace zipml

using namespace zipml;

extern "C" int zipml_sgd_epoch(void *stream, const void *packed1_dev, const void *packed2_dev,
                               const float *levels_dev, const uint16_t *grid_idx_dev,
                               float grid_lo, float grid_step, int grid_max, const float *b_dev,
                               int64_t n, int64_t d, int bits, float *x_dev, int64_t batch,
                               float lr, int grad_bits, int model_bits, uint64_t seed,
                               uint32_t epoch, int flags, void *workspace_dev,
                               size_t workspace_bytes)
{
    const int64_t steps = (batch > 0 && n > 0 && n % batch == 0) ? n / batch : 0;
    return run_sgd(stream, packed1_dev, packed2_dev, nullptr, nullptr, levels_dev, grid_idx_dev,
                   grid_lo, grid_step, grid_max, b_dev, n, d, bits, x_dev, batch, lr, 0.0f, grad_bits,
                   model_bits, seed, epoch, flags, 0, steps, nullptr, nullptr, nullptr, nullptr, nullptr,
                   workspace_dev, workspace_bytes);
}

extern "C" int zipml_sgd_epoch_l2(void *stream, const void *packed1_dev, const void *packed2_dev,
                                  const float *levels_dev, const float *b_dev, int64_t n, int64_t d,
                                  int bits, float *x_dev, int64_t batch, float lr, float l2,
                                  int flags, void *workspace_dev, size_t workspace_bytes)
{
    const int64_t steps = (batch > 0 && n > 0 && n % batch == 0) ? n / batch : 0;
    return run_sgd(stream, packed1_dev, packed2_dev, nullptr, nullptr, levels_dev, nullptr, 0.0f, 0.0f,
                   0, b_dev, n, d, bits, x_dev, batch, lr, l2, 0, 0, 0, 0, flags, 0, steps, nullptr,
                   nullptr, nullptr, nullptr, nullptr, workspace_dev, workspace_bytes);
}

extern "C" int zipml_sgd_epoch_prox(void *stream, const void *packed1_dev, const void *packed2_dev,
                                    const float *levels_dev, const float *b_dev, int64_t n, int64_t d,
                                    int bits, float *x_dev, int64_t batch, float lr, float l2,
                                    int prox, float prox_coef, int flags, void *workspace_dev,
                                    size_t workspace_bytes)
{
    const int64_t steps = (batch > 0 && n > 0 && n % batch == 0) ? n / batch : 0;
    return run_sgd(stream, packed1_dev, packed2_dev, nullptr, nullptr, levels_dev, nullptr, 0.0f, 0.0f,
                   0, b_dev, n, d, bits, x_dev, batch, lr, l2, 0, 0, 0, 0, flags, 0, steps, nullptr,
                   nullptr, nullptr, nullptr, nullptr, workspace_dev, workspace_bytes, prox, prox_coef);
}

extern "C" int zipml_sgd_epoch_avg(void *stream, const void *packed1_dev, const void *packed2_dev,
                                   const void *packed1s_dev, const void *packed2s_dev,
                                   const float *levels_dev, const float *b_dev, int64_t n, int64_t d,
                                   int bits, float *x_dev, int64_t batch, float lr, float l2,
                                   int flags, void *workspace_dev, size_t workspace_bytes)
{
    if (!packed1s_dev || !packed2s_dev) return ZIPML_EINVAL;
    const int64_t steps = (batch > 0 && n > 0 && n % batch == 0) ? n / batch : 0;
    return run_sgd(stream, packed1_dev, packed2_dev, packed1s_dev, packed2s_dev, levels_dev, nullptr,
                   0.0f, 0.0f, 0, b_dev, n, d, bits, x_dev, batch, lr, l2, 0, 0, 0, 0, flags, 0, steps,
                   nullptr, nullptr, nullptr, nullptr, nullptr, workspace_dev, workspace_bytes);
}

// The epoch on the compact record of the two sample-major copies (zipml_sgd_rows_compact.h).
extern "C" int zipml_sgd_epoch_compact(void *stream, const void *compact_dev, const float *levels_dev,
                                       const float *b_dev, int64_t n, int64_t d, int bits, float *x_dev,
                                       int64_t batch, float lr, void *workspace_dev, size_t workspace_bytes)
{
    if (!compact_dev || !levels_dev || !b_dev || !x_dev) return ZIPML_EINVAL;
    if (n <= 0 || d <= 0 || !valid_bits(bits) || batch <= 0 || n % batch != 0) return ZIPML_EINVAL;
    if (n > (int64_t)1 << 40 || d > (1 << 24)) return ZIPML_EINVAL;
    if (!aligned16(compact_dev) || !aligned16(levels_dev) || !aligned16(b_dev) || !aligned16(x_dev) ||
        !aligned16(workspace_dev))
        return ZIPML_EALIGN;
    if (!workspace_dev || workspace_bytes < zipml_workspace_bytes(n, d, bits, batch, 0)) return ZIPML_EWORKSPACE;
    const Layout lay = make_layout(n, d, bits);
    const int NKB = (int)((lay.d32 + 1) / 2);
    // built for 8-bit codes (where the record saves most), minibatches that the sample owners take,
    // and 9 to 32 blocks of 64 features (a wave keeps copy 1 of its two or four blocks of a tile in LDS)
    if (bits != 8 || batch < Workspace::kRowsMinBatch || batch % 64 != 0 || NKB <= kWaves || NKB > 4 * kWaves)
        return ZIPML_EUNSUPPORTED;
    hipStream_t s = entry_stream(stream);
    int cus = 0, lds = 0;
    if (int rc = device_limits(cus, lds)) return rc;
    const size_t shmem = rows_compact_lds_bytes(NKB);
    if (shmem > (size_t)lds) return ZIPML_EUNSUPPORTED;
    int wgs = std::min(cus, Workspace::kMaxRowsWgs);
    if (const long long v = knob(ZIPML_KNOB_ROWS_WORKGROUPS); v >= 1 && v <= Workspace::kMaxRowsWgs) wgs = (int)v;
    unsigned char *wsb = (unsigned char *)workspace_dev;
    float *rows = (float *)(wsb + Workspace::sgd_bytes(batch) + (size_t)round_up(d, 64) * 4);
    RowsArgs r{};
    r.p1 = nullptr;
    r.p2 = (const uint32_t *)compact_dev;
    r.b = b_dev;
    r.x = x_dev;
    r.dl = rows;
    r.mid = rows + (size_t)NKB * 64;
    r.part = rows + (size_t)2 * NKB * 64;
    r.n_pad = lay.n_pad;
    r.n32 = lay.n32;
    r.d = (int)d;
    r.d32 = (int)lay.d32;
    r.NKB = NKB;
    r.B = batch;
    r.step0 = 0;
    r.nsteps = (int)(n / batch);
    r.lr = lr;
    r.status = (int *)(wsb + Workspace::kStatus);
    r.sync = (uint32_t *)(wsb + Workspace::kSync);
    r.even = (const int *)(wsb + Workspace::kEven);
    r.spin_limit = kSpinLimit;
    if (const long long v = knob(ZIPML_KNOB_SPIN_LIMIT); v >= 0 && v <= (long long)kSpinLimit) r.spin_limit = (uint32_t)v;
    const void *kern = NKB <= 2 * kWaves ? (const void *)k_sgd_rows_compact<2> : (const void *)k_sgd_rows_compact<4>;
    if (HIP_FAILED(hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem)))
        return ZIPML_ELAUNCH;
    hipLaunchKernelGGL(k_sgd_prepare, dim3(Workspace::kEvenBlocks + 1), dim3(kPrepThreads), 0, s, r.status, r.sync,
                       (uint64_t *)(wsb + Workspace::kAcc), 0, 1, levels_dev, r.x, r.d, 256, (double *)nullptr,
                       (int *)(wsb + Workspace::kEven), const_cast<float *>(r.dl), const_cast<float *>(r.mid),
                       NKB * 64, 128.0f);
    if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    void *params[] = {&r};
    return launch_resident(kern, wgs, params, shmem, s);
}

extern "C" int zipml_debug_step(void *stream, const void *packed1_dev, const void *packed2_dev,
                                const float *levels_dev, const uint16_t *grid_idx_dev,
                                float grid_lo, float grid_step, int grid_max, const float *b_dev,
                                int64_t n, int64_t d, int bits, float *x_dev, int64_t batch,
                                float lr, int grad_bits, int model_bits, uint64_t seed,
                                uint32_t epoch, int64_t step, int flags, int32_t *model_codes_dev,
                                int32_t *acc_dev, float *r_dev, float *g_dev,
                                int32_t *grad_codes_dev, void *workspace_dev,
                                size_t workspace_bytes)
{
    return run_sgd(stream, packed1_dev, packed2_dev, nullptr, nullptr, levels_dev, grid_idx_dev,
                   grid_lo, grid_step, grid_max, b_dev, n, d, bits, x_dev, batch, lr, 0.0f, grad_bits,
                   model_bits, seed, epoch, flags, step, 1, model_codes_dev, acc_dev, r_dev, g_dev, grad_codes_dev,
                   workspace_dev, workspace_bytes);
}

// ---------------------------------------------------------------------------------------------
// zipml_sgd_epoch for callers that cannot allocate: the workspace is a fixed array inside the
// library's code object.  `scratch` below is, in host code, only a stand-in for the symbol: its
// device address differs from device to device and is looked up once per device with
// hipGetSymbolAddress; everything after that uses the address found, never the name.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[ZIPML_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device; null: not looked up yet

int static_scratch(void **out)
{
    int dev = 0;
    if (HIP_FAILED(hipGetDevice(&dev))) return ZIPML_ELAUNCH;
    if (dev < 0 || dev >= kMaxDevices) return ZIPML_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (HIP_FAILED(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) || !p) return ZIPML_ELAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ZIPML_OK;
}
}  // namespace

extern "C" int zipml_sgd_epoch_static(void *stream, const void *packed1_dev, const void *packed2_dev,
                                      const float *levels_dev, const uint16_t *grid_idx_dev,
                                      float grid_lo, float grid_step, int grid_max,
                                      const float *b_dev, int64_t n, int64_t d, int bits,
                                      float *x_dev, int64_t batch, float lr, int grad_bits,
                                      int model_bits, uint64_t seed, uint32_t epoch, int flags,
                                      int *status_dev)
{
    if (!status_dev || (reinterpret_cast<uintptr_t>(status_dev) & 3u)) return ZIPML_EINVAL;
    const size_t need = zipml_workspace_bytes(n, d, bits, batch, 0);
    if (need == 0) return ZIPML_EINVAL;
    if (need > (size_t)ZIPML_STATIC_WORKSPACE_BYTES) {
        fprintf(stderr, "libzipml: zipml_sgd_epoch_static: this shape needs %zu bytes of workspace, the "
                        "built-in one has %zu; use zipml_sgd_epoch with a workspace of the caller's\n",
                need, (size_t)ZIPML_STATIC_WORKSPACE_BYTES);
        return ZIPML_EWORKSPACE;
    }
    void *ws = nullptr;
    if (int rc = static_scratch(&ws)) return rc;
    const int64_t steps = (batch > 0 && n > 0 && n % batch == 0) ? n / batch : 0;
    return run_sgd(stream, packed1_dev, packed2_dev, nullptr, nullptr, levels_dev, grid_idx_dev,
                   grid_lo, grid_step, grid_max, b_dev, n, d, bits, x_dev, batch, lr, 0.0f, grad_bits,
                   model_bits, seed, epoch, flags, 0, steps, nullptr, nullptr, nullptr, nullptr, nullptr,
                   ws, (size_t)ZIPML_STATIC_WORKSPACE_BYTES, ZIPML_PROX_NONE, 0.0f, status_dev);
}

extern "C" int zipml_sgd_status(void *stream, const void *workspace_dev, size_t workspace_bytes)
{
    if (!workspace_dev || workspace_bytes < 4096) return ZIPML_EWORKSPACE;
    int st = 0;
    hipStream_t s = entry_stream(stream);
    if (HIP_FAILED(hipMemcpyAsync(&st, (const unsigned char *)workspace_dev + Workspace::kStatus,
                                  sizeof(int), hipMemcpyDeviceToHost, s)))
        return ZIPML_ELAUNCH;
    if (HIP_FAILED(hipStreamSynchronize(s))) return ZIPML_ELAUNCH;
    return st;
}
