// Step loop of the epoch kernel on the matrix cores: evenly spaced levels, fp32 model, 2-, 4- or
// 8-bit codes (included by zipml_sgd.hip; uses its SgdArgs / Lds / exchange-word helpers).
//
// With evenly spaced levels a value is lo_j + code * delta_j = mid_j + (code - off) * delta_j
// (off = 128 for 8-bit codes, which re-centres them into a signed byte, else 0), so both passes of
// eq. (5), Sec. 2.2, are integer-weighted sums:
//     z_i = sum_j mid_j x_j + sum_j (code2_ij - off) y_j,        y_j = delta_j x_j,
//     g_j = (mid_j sum_i r_i + delta_j sum_i (code1_ij - off) r_i) / B.
// The vectors y and r are turned into 32-bit fixed point (one common power-of-two scale per step)
// and split into four signed base-256 digits; the packed codes, expanded to one byte each, are the
// other operand of v_mfma_i32_16x16x64_i8:
//     dot pass       C[digit][sample]  += Ydigits[digit][64 features] * codes2[64 features][sample]
//     gradient pass  C[digit][feature] += Rdigits[digit][64 samples]  * codes1[64 samples][feature]
// Only 4 of the 16 rows of the digit operand are used; the instruction still does in one issue
// what takes 128 convert + multiply-add instructions per lane on the vector ALU.  All sums are
// exact integers: the result does not depend on the order of anything, and the only roundings are
// the conversions of y_j, r_i to fixed point (relative 2^-29 of the largest element) and of the
// sums back to fp32.
//
// Operand layout of the instruction (checked against a host reference on the device):
//   A: lane l holds row l%16, k = 16*(l/16) .. +15 (16 bytes);  B: lane l holds column l%16, same k;
//   C: lane l holds column l%16, rows 4*(l/16) .. +3.
// A lane's 16 code bytes come from 16*BITS/8 packed bytes; code_slot() says which byte a code of
// the packed unit lands in, and the digit operands are laid out in LDS with the same map.
//
// The vector ALU is left with bookkeeping, and at small batches that is what a step costs besides
// the exchange, so only as many waves work in the loop as have samples or features to look after
// (4 of the 8 when the batch has at most 256 samples; the others only keep the workgroup barriers
// company), and everything uniform is done in fp32.
#pragma once
#include "zipml_mfma_ops.h"

namespace zipml {

// LDS bytes of the matrix-core path for a plan.
__host__ __device__ inline size_t mfma_lds_bytes(int GQ, int64_t batch, int pairs)
{
    const size_t KB = (size_t)(GQ + 1) / 2;
    return KB * 256 + (size_t)pairs * (size_t)(batch / 64) * 256 + (size_t)4 * 32 * GQ * 8 + 512;
}

constexpr int kRefresh = 16;   // steps between exact refreshes of the magnitude bounds

// Exchange through tagged stores (a.xstore), for launches in which the number of exchange words
// times the number of workgroups is large.  One atomic per (workgroup, sample) is what the
// device-wide exchange costs then: the memory side completes some 15-25 atomics per ns, and the
// tomography shape has 65,536 of them per step.  Plain stores and loads are far cheaper, so the
// sums are formed in two trips instead:
//   1. a workgroup STORES its partial sums, one 64-bit word per sample in its own row
//      part[u & 1][workgroup][word]; a word carries a 16-bit tag of the step above the 48-bit
//      fixed-point value, so one store delivers value and arrival (no counts, nothing to clear
//      between steps: a stale word has another tag);
//   2. the words are dealt out in pieces of eight (64 bytes) to "reducer" workgroups; a reducer
//      polls its piece in every row, adds the W values (integers: exact, any order) and stores the
//      sums, tagged the same way, to res[u & 1][word];
//   3. every thread polls the result words of its own samples.
// Two buffers alternate (per replica, when the chunks of a minibatch are shared out: a replica's
// exchanges are its own).  A workgroup writes row words of step u only after it has finished step
// u-1, for which it needed results that every reducer published after its reads of step u-2; a
// reducer writes results of step u after it has seen every workgroup's words of step u, which
// each wrote after reading the results of step u-2.  So no word is overwritten while someone may
// still read it.  The preparation launch clears both arrays (a stale tag of an earlier call could
// otherwise match).
constexpr int kPiece = 8;                                  // exchange words per reducer piece
__device__ __forceinline__ uint64_t tag_word(uint32_t tag, long long v)
{
    return ((uint64_t)tag << 48) | ((uint64_t)v & 0x0000FFFFFFFFFFFFull);
}
__device__ __forceinline__ long long tagged_value(uint64_t word)
{
    return (long long)(word << 16) >> 16;                  // sign-extends the 48-bit field
}
constexpr int64_t kWatchFirst = 32768;   // exchange words x workgroups from which a wave polls one word first

// KB: 64-feature blocks per workgroup (1: GQ <= 2, 2: GQ == 4).
// NC: 1 = the estimator of eq. (5), g = mean_i Q1(a_i) (Q2(a_i)^T x - b_i);
//     2 = its symmetrised form (Supp. B.2, footnote), 1/2 mean_i [Q1 (Q2^T x - b) + Q2 (Q1^T x - b)]: a
//     second pair of packed arrays holds copy 1 sample-major and copy 2 feature-major, both
//     pairs go through the same two passes at the same model, with one exchange for both.
// REP: the chunks of a minibatch are shared out over replicas of the workgroups (a.R > 1).
// XM: 0 = the plain loop (exchange through atomics), 1 = exchange through tagged stores,
//     2 = the plain loop that also writes the residuals and the gradient of its steps to the
//     debug outputs (zipml_debug_step with ZIPML_SGD_PRODUCTION).  Instantiations of their own, so
//     that neither costs the plain loop registers.
template <int BITS, int UPT, int KB, int NC, bool REP, int XM>
__device__ __forceinline__ void sgd_steps_mfma(const SgdArgs &a, const Lds &L, unsigned char *mf)
{
    constexpr bool kDbg = XM == 2;
    constexpr int HW = BITS / 2;                       // packed dwords per lane operand
    constexpr int kSlots = KB == 1 ? UPT : (UPT + 3) / 4;   // groups of four 16-sample tiles per wave
    constexpr int kTiles = 4 * kSlots;                 // 16-sample tiles per wave, at most
    constexpr int kNG = UPT == 1 ? 4 : 2 * UPT;        // gradient instructions per wave, at most
    // Small steps hold two steps of packed data in registers (the loads need more than a step to
    // arrive); large steps are long enough for loads issued one step ahead, and need the registers.
    constexpr bool kDouble = UPT <= 2 && NC == 1;
    constexpr int kT2 = kDouble ? kTiles : 1, kG2 = kDouble ? kNG : 1;
    constexpr int kBpt = UPT;                          // samples per thread in the residual phase
    constexpr float kOff = BITS == 8 ? 128.0f : 0.0f;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;
    const int W = a.W, GQ = a.GQ, CW = 32 * GQ, B = a.B;
    const int w = blockIdx.x % W;                       // feature block of this workgroup
    const int R = REP ? a.R : 1, rep = REP ? blockIdx.x / W : 0;   // replicas (see below), and which one this is
    const int j0 = w * CW;
    const int ngroups = (a.d32 - w * GQ) < GQ ? (a.d32 - w * GQ) : GQ;
    const int ntile = B / 16, NKS = B / 64;
    const int FT = 2 * GQ;                              // 16-feature tiles (2, 4 or 8)
    const int nw = (UPT == 1 && B <= 256 && FT <= 4) ? 4 : kWaves;   // waves that work in the loop
    const int nthr = nw * kWave;
    const int KSS = nw / FT;                            // waves that share a feature tile
    const int g_ft = wave % FT, g_kh = wave / FT;
    const bool owner = g_kh == 0 && lane < 16;          // this lane updates feature 16*g_ft + lane
    const int oc = 16 * g_ft + n16;                     // that feature, inside the workgroup
    float *const xs = L.xs;
    // A minibatch of a.chunks * B samples is taken in chunks of B: every chunk has its own
    // exchange, the model is updated after the last one.  The chunks of a minibatch do not depend
    // on each other, so R replicas of the W workgroups (each with its own exchange buffers and its
    // own, identical copy of the model) take every R-th chunk each: replica `rep` takes the chunks
    // rep, rep + R, ... of every minibatch, C = a.chunks / R of them, which are R chunks apart
    // through the whole epoch.  After its last chunk of a minibatch a workgroup hands its share of
    // the gradient to the R - 1 workgroups that own the same features (exchange_gradient below);
    // all add the R shares in the same order, so the copies of the model stay identical.
    // u counts this replica's chunks through the epoch; chunk u is chunk u * R + rep of the data.
    const int C = a.chunks / R;
    const int64_t u_begin = a.step0 * C, u_end = (a.step0 + a.nsteps) * C;
    const int nwords = NC * B + 2;                      // exchange words of a chunk: sums, 2 side words
    const bool xstore = XM == 1 && nw == kWaves;        // exchange through tagged stores (see above; all waves take part)
    const int xrow = a.xrow;                            // words per row of part[][] and of res[] (multiple of kPiece)
    const int npieces = (nwords + kPiece - 1) / kPiece;
    // (every replica has its own rows and results: [2][W][xrow] and [2][xrow] words)
    uint64_t *const xbase = a.xpart + (size_t)rep * ((size_t)2 * (W + 1) * xrow);
    const int clr_per = (nwords + W - 1) / W;           // words of a later step that this workgroup clears
    const int clr_lo = w * clr_per, clr_hi = clr_lo + clr_per < nwords ? clr_lo + clr_per : nwords;
    uint64_t *const acc_base = a.acc + (size_t)rep * Workspace::kAccBuffers * a.acc_words;
    const uint32_t *const p2base[2] = {a.p2, a.p2s}, *const p1base[2] = {a.p1, a.p1s};

    // ---- LDS of this path
    int8_t *const ydig = (int8_t *)mf;                              // [KB][4 digits][4 q][16]
    int8_t *const rdig = ydig + KB * 256;                           // [NC][NKS][4 digits][4 q][16]
    long long *const gpart = (long long *)(rdig + (size_t)NC * NKS * 256);   // [4][CW]
    unsigned char *misc = (unsigned char *)(gpart + 4 * CW);
    float *const cqs = (float *)misc;                               // [8] per tile: sum_j mid_j x_j
    float *const bws = (float *)(misc + 32);                        // [8] sum_j maxabs(L_j)|x_j|
    int *const ymx = (int *)(misc + 64);                            // [8] max_j |Y_j|
    float *const wmax = (float *)(misc + 96);                       // [8] per wave max_i |r_i|
    float *const wsum = (float *)(misc + 128);                      // [8] per wave sum_i r_i
    float *const side = (float *)(misc + 160);                      // [2] decoded side words, [1] largest |residual| of all replicas

    for (int e = tid; e < KB * 256 + NC * NKS * 256; e += kThreads) ydig[e] = 0;
    if (tid < 8) { cqs[tid] = 0.0f; bws[tid] = 0.0f; ymx[tid] = 0; wmax[tid] = 0.0f; wsum[tid] = 0.0f; }
    lds_barrier();

    if (wave >= nw) {
        // nothing to look after: meet the others at their barriers, step by step
        for (int64_t u = u_begin; u < u_end; ++u) {
            lds_barrier();
            if (wave == kWaves - 1) {
                // clear this workgroup's share of the exchange words of step t+2 (see zipml_sgd.hip for why now)
                uint64_t *nxt = acc_base + (size_t)((u + 2) & 3) * a.acc_words;
                for (int i = clr_lo + lane; i < clr_hi; i += kWave) store_dev(nxt + i, (uint64_t)0);
                vm_wait_all();
            }
            if (xstore)
                for (int pc = w; pc < npieces; pc += W) lds_barrier();   // (the reducer's, see below)
            lds_barrier();
            lds_barrier();
            if (KSS > 1) lds_barrier();
        }
        lds_barrier();
        return;
    }

    // ---- bounds that fix the fixed-point scale of a step; every workgroup computes the same
    // numbers in the same order.  beta_hat >= sum_j maxabs(L_j)|x_j| bounds every partial and full
    // dot product; ymax_hat >= max_j |y_j| keeps the digits of y inside 32 bits.  Both are exact
    // at launch, grow every step by a bound on the model's change (|dx_j| <= lr (maxabs(L_j) max_i
    // |r_i| + c |x_j|)), and are refreshed from exact per-workgroup values every kRefresh steps.
    float beta_hat = (float)a.bound[0] * 1.00001f;
    const float lambda = (float)a.bound[1] * 1.00001f;   // sum_j maxabs(L_j)^2
    float ymax_hat = (float)a.bound[2] * 1.00001f;
    const float mu = (float)a.bound[3] * 1.00001f;       // max_j delta_j maxabs(L_j)
    const float lr_abs = fabsf(a.lr) * 1.00001f, l2_abs = fabsf(a.l2) * 1.00001f;
    auto scale_of = [&]() {
        const int k1 = scale_exponent(beta_hat, 42), k2 = scale_exponent(ymax_hat, 29);
        return k1 < k2 ? k1 : k2;
    };
    int ky = scale_of();
    int ky_pub = ky;                                   // the scale the sums in flight were published with

    // ---- owner lanes: per-feature constants, and where the digits of y_j go
    const float o_lo = owner ? L.los[oc] : 0.0f, o_dl = owner ? L.dls[oc] : 0.0f;
    const float o_mid = o_lo + kOff * o_dl;
    const float o_maxl = fmaxf(fabsf(o_lo), fabsf(o_lo + o_dl * (float)((1 << BITS) - 1))) * 1.00001f;
    const bool o_live = owner && (j0 + oc < a.d);
    int y_pos = 0;
    {
        int half, byte;
        code_slot<BITS>(oc & 31, half, byte);
        const int gq = oc >> 5;
        y_pos = ((gq >> 1) * 4) * 64 + (2 * (gq & 1) + half) * 16 + byte;   // digit plane 0
    }
    // y_j -> digits in LDS, and the per-tile sums the next exchange needs (all 64 lanes of an
    // owner wave take part in the row reductions; only lanes 0..15 hold real values)
    auto refresh_y = [&](float x, int kscale, bool with_bounds) {
        const float y = o_dl * x;
        const int Y = owner ? __float2int_rn(ldexpf(y, kscale)) : 0;
        if (owner) store_digits(ydig + y_pos, signed_digits(Y));
        const float cq = row_reduce_dpp(owner ? o_mid * x : 0.0f, [](float p, float q) { return p + q; });
        if (lane == 0) cqs[g_ft] = cq;
        if (with_bounds) {
            const float bw = row_reduce_dpp(owner ? o_maxl * fabsf(x) : 0.0f, [](float p, float q) { return p + q; });
            const int amx = row_reduce_dpp(Y < 0 ? -Y : Y, [](int p, int q) { return p > q ? p : q; });
            if (lane == 0) { bws[g_ft] = bw; ymx[g_ft] = amx; }
        }
    };
    float x_own = owner ? xs[oc] : 0.0f;               // the owner lane keeps its feature's weight
    if (g_kh == 0) refresh_y(x_own, ky, true);

    // ---- packed data held in registers; the addresses advance by a fixed stride per step
    const int64_t step_dwords = (int64_t)R * B * BITS;  // both copies: B samples x BITS dwords per group,
                                                        // R chunks from one chunk of this replica to its next
    const int64_t row_begin = (u_begin * R + rep) * B;  // first sample of this replica's first chunk
    uint32_t c2cur[NC][kTiles][KB][HW], c2nxt[kT2][KB][HW], c1[NC][kNG][HW], c1nxt[kG2][HW];
    const uint32_t *p2ptr[NC][kTiles][KB], *p1ptr[NC][kNG];
    bool p2ok[kTiles][KB], p1ok[kNG];
    float bnext[kBpt], bfut[kBpt];
#pragma unroll
    for (int ti = 0; ti < kTiles; ++ti) {
        const int tile = wave + nw * ti;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const int gq = 2 * kb + (q4 >> 1);
            p2ok[ti][kb] = tile < ntile && gq < ngroups;
            const int64_t row = row_begin + 16 * tile + n16;
            const int64_t g = (int64_t)w * GQ + gq;
#pragma unroll
            for (int cc = 0; cc < NC; ++cc)
                p2ptr[cc][ti][kb] = p2ok[ti][kb] ? p2base[cc] + (g * a.nb64 * 64 + row) * BITS + (q4 & 1) * HW
                                                 : p2base[cc];
        }
    }
#pragma unroll
    for (int m = 0; m < kNG; ++m) {
        const int ks = g_kh + KSS * m;
        const int gq = g_ft >> 1, cin = 16 * (g_ft & 1) + n16;
        p1ok[m] = ks < NKS && gq < ngroups;
        const int64_t g = (int64_t)w * GQ + gq;
        const int64_t rg = row_begin / 32 + 2 * ks + (q4 >> 1);
#pragma unroll
        for (int cc = 0; cc < NC; ++cc)
            p1ptr[cc][m] = p1ok[m] ? p1base[cc] + ((g * a.n32 + rg) * 32 + cin) * BITS + (q4 & 1) * HW
                                   : p1base[cc];
    }
    // loads of the step `ahead` steps after the one the pointers stand at
    auto load_dot = [&](int cc, int ahead, auto &dst) {
#pragma unroll
        for (int ti = 0; ti < kTiles; ++ti)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const uint32_t *q = static_cast<const uint32_t *>(
                    __builtin_assume_aligned(p2ptr[cc][ti][kb] + ahead * step_dwords, 4 * HW));
                if (p2ok[ti][kb]) {
#pragma unroll
                    for (int k = 0; k < HW; ++k) dst[ti][kb][k] = q[k];
                }
            }
    };
    auto load_grad = [&](int cc, int ahead, auto &dst) {
#pragma unroll
        for (int m = 0; m < kNG; ++m) {
            const uint32_t *q = static_cast<const uint32_t *>(
                __builtin_assume_aligned(p1ptr[cc][m] + ahead * step_dwords, 4 * HW));
            if (p1ok[m]) {
#pragma unroll
                for (int k = 0; k < HW; ++k) dst[m][k] = q[k];
            }
        }
    };
    auto load_labels = [&](int64_t uu, float (&dst)[kBpt]) {
#pragma unroll
        for (int k = 0; k < kBpt; ++k) {
            const int i = tid + k * nthr;
            if (i < B) dst[k] = a.b[(uu * R + rep) * B + i];
        }
    };
    // operands that are never loaded multiply digit rows that are zero; give them a value anyway
#pragma unroll
    for (int ti = 0; ti < kTiles; ++ti)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int k = 0; k < HW; ++k) {
#pragma unroll
                for (int cc = 0; cc < NC; ++cc) c2cur[cc][ti][kb][k] = 0u;
                if constexpr (kDouble) c2nxt[ti][kb][k] = 0u;
            }
#pragma unroll
    for (int m = 0; m < kNG; ++m)
#pragma unroll
        for (int k = 0; k < HW; ++k) {
#pragma unroll
            for (int cc = 0; cc < NC; ++cc) c1[cc][m][k] = 0u;
            if constexpr (kDouble) c1nxt[m][k] = 0u;
        }
#pragma unroll
    for (int k = 0; k < kBpt; ++k) bnext[k] = bfut[k] = 0.0f;
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) {
        load_dot(cc, 0, c2cur[cc]);
        load_grad(cc, 0, c1[cc]);
    }
    if constexpr (kDouble) {
        if (u_begin + 1 < u_end) load_dot(0, 1, c2nxt);
    }
    load_labels(u_begin, bnext);

    // where the digits of this thread's residuals go: sample i -> k-step i/64, q, byte
    int r_pos[kBpt];
#pragma unroll
    for (int k = 0; k < kBpt; ++k) {
        const int i = tid + k * nthr;
        int half, byte;
        code_slot<BITS>(i & 31, half, byte);
        r_pos[k] = ((i >> 6) * 4) * 64 + (2 * ((i >> 5) & 1) + half) * 16 + byte;
    }

    bool dead = false;
#ifdef ZIPML_PHASE_TIMING
    long long prof_[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = wall_clock64();
#endif

    float rmax_step = 0.0f, gsum = 0.0f;
    int64_t t = a.step0;                                        // minibatch step
    int chunk = 0;
    for (int64_t u = u_begin; u < u_end; ++u) {
        const bool first = chunk == 0, last = chunk == C - 1;
        uint64_t *const acc = acc_base + (size_t)(u & 3) * a.acc_words;
        const uint32_t xtag = ((uint32_t)(u + 1) & 0x7FFFu) | 0x8000u;
        uint64_t *const xpart = xbase + (size_t)(u & 1) * ((size_t)W * xrow);
        uint64_t *const xres = xbase + (size_t)2 * W * xrow + (size_t)(u & 1) * xrow;
        const bool side_step = first && (t % kRefresh) == 0;   // bounds travel with this exchange
        const bool side_next = last && ((t + 1) % kRefresh) == 0;
        ZIPML_TICK(7);
        lds_barrier();          // digits of y and the per-tile sums of the current model
        ZIPML_TICK(0);
        if (REP && first && u > u_begin) {
            // the model has just moved by the gradient of all replicas: grow the bounds by the
            // largest residual any of them saw (left in LDS by the owner waves)
            const float rall = side[2];
            beta_hat += lr_abs * (lambda * rall + l2_abs * beta_hat);
            ymax_hat += lr_abs * (mu * rall + l2_abs * ymax_hat);
            ky = scale_of();
            rmax_step = 0.0f;
        }

        // Dot pass of chunk uu at the model whose digits are in LDS, its partial sums into the
        // exchange, then the requests for the data of later chunks.  (A function of the chunk so that
        // the development build -DZIPML_STALE_DOT_EXPERIMENT can publish chunk u + 1 from the OLD
        // model before the gradient pass of chunk u: a one-step-delayed SGD, not the paper's, which
        // bounds from above what taking the gradient pass and the update off the path between two
        // exchanges could gain.  Measured on the dense 8-bit shape: nothing, 2.95 against 2.99 us per
        // step -- a step is the sum of its phases, and reading the exchange words, a device-scope load
        // of some 0.6 us, stays on the path however early the sums were published.)
        auto dot_and_publish = [&](int64_t uu, bool pub_side) __attribute__((always_inline)) {
        uint64_t *const pub_acc = acc_base + (size_t)(uu & 3) * a.acc_words;
        const uint32_t pub_xtag = ((uint32_t)(uu + 1) & 0x7FFFu) | 0x8000u;
        uint64_t *const pub_xmine = xbase + (size_t)(uu & 1) * ((size_t)W * xrow) + (size_t)w * xrow;
        ky_pub = ky;
        // ============ dot pass: one instruction per (16 samples, 64 features)
        {
            // what every sample of this workgroup gets on top of sum_j (code - off) * Y_j
            const float4 c0 = *reinterpret_cast<const float4 *>(cqs);
            const float4 c1v = *reinterpret_cast<const float4 *>(cqs + 4);
            const float cq = ((c0.x + c0.y) + (c0.z + c0.w)) + ((c1v.x + c1v.y) + (c1v.z + c1v.w));
            // cq * 2^ky as an integer (|.| < 2^43) without fp64: high part, then the exact rest
            const float sc = ldexpf(cq, ky - 24), sc_hi = truncf(sc);
            const long long kconst = ((long long)(int)sc_hi << 24) + (long long)__float2int_rn(ldexpf(sc - sc_hi, 24));
            // Four sample tiles share one accumulator: the digits of tile slot s sit in rows
            // 4s..4s+3 of its digit operand (zeros elsewhere), so its sums land in lanes
            // 16s..16s+15 and one combine / one atomic instruction serves all 64 lanes.
            const v4i zero = {0, 0, 0, 0};
            v4i afull[KB];
#pragma unroll
            for (int kb = 0; kb < KB; ++kb)
                afull[kb] = *reinterpret_cast<const v4i *>(ydig + (kb * 4 + (n16 & 3)) * 64 + q4 * 16);
#pragma unroll
            for (int cc = 0; cc < NC; ++cc) {
#pragma unroll
                for (int gi = 0; gi < kSlots; ++gi) {
                    if (wave + nw * 4 * gi < ntile) {
                        v4i c = {0, 0, 0, 0};
#pragma unroll
                        for (int sl = 0; sl < 4; ++sl) {
#pragma unroll
                            for (int kb = 0; kb < KB; ++kb) {
                                const v4i as = (n16 >> 2) == sl ? afull[kb] : zero;
                                c = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                                    as, expand_codes<BITS>(c2cur[cc][4 * gi + sl][kb]), c, 0, 0, 0);
                            }
                        }
                        const int tile = wave + nw * (4 * gi + q4);
                        if (tile < ntile) {
                            if (xstore) store_dev(pub_xmine + cc * B + 16 * tile + n16, tag_word(pub_xtag, combine_digits(c) + kconst));
                            else add_dev(pub_acc + cc * B + 16 * tile + n16, pack_int(combine_digits(c) + kconst));
                        }
                    }
                }
            }
            ZIPML_TICK(2);
            if (pub_side && wave == 0 && lane < 2) {
                // side words: this workgroup's share of the two bounds, rounded up
                float bw = 0.0f;
                int mx = 0;
                for (int f = 0; f < FT; ++f) {
                    bw += bws[f];
                    mx = ymx[f] > mx ? ymx[f] : mx;
                }
                const long long v = lane == 0 ? __double2ll_ru(ldexp((double)bw, ky)) + 1 : (long long)mx;
                if (xstore) store_dev(pub_xmine + NC * B + lane, tag_word(pub_xtag, v));
                else add_dev(pub_acc + NC * B + lane, pack_int(v));
            }
        }
        // The last wave of every workgroup clears its share of the exchange words of step t+2 (see
        // zipml_sgd.hip for why that is the right moment and why no wait is needed here); with
        // idle waves around, one of them does it instead.
        if (!xstore && nw == kWaves && wave == kWaves - 1) {
            uint64_t *nxt = acc_base + (size_t)((uu + 2) & 3) * a.acc_words;
            for (int i = clr_lo + lane; i < clr_hi; i += kWave) store_dev(nxt + i, (uint64_t)0);
            if (!(tid < B)) vm_wait_all();
        }
        ZIPML_TICK(11);
        // Rotate copy 2 and request what later steps need, now: the loads travel while the
        // exchange is under way.  (A wave's memory operations complete in order and the compute
        // unit's memory pipeline keeps that order too, so the poll below cannot return before
        // these loads have; issued anywhere else their latency would add to the exchange's
        // instead of hiding behind it.)
#pragma unroll
        for (int ti = 0; ti < kTiles; ++ti)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                if constexpr (kDouble) {
#pragma unroll
                    for (int k = 0; k < HW; ++k) c2cur[0][ti][kb][k] = c2nxt[ti][kb][k];
                }
#pragma unroll
                for (int cc = 0; cc < NC; ++cc) p2ptr[cc][ti][kb] += step_dwords;   // now at step t+1
            }
        if constexpr (kDouble) {
            if (uu + 2 < u_end) load_dot(0, 1, c2nxt);
            if (uu + 1 < u_end) load_grad(0, 1, c1nxt);
        } else {
            if (uu + 1 < u_end) {
#pragma unroll
                for (int cc = 0; cc < NC; ++cc) load_dot(cc, 0, c2cur[cc]);
            }
        }
        if (uu + 1 < u_end) load_labels(uu + 1, bfut);
        ZIPML_TICK(1);
        };
#ifdef ZIPML_STALE_DOT_EXPERIMENT
        if (!(XM == 0 && NC == 1 && !REP && C == 1) || u == u_begin) dot_and_publish(u, side_step);
#else
        dot_and_publish(u, side_step);
#endif

        // ============ tagged-store exchange, second trip: this workgroup's pieces of the sums
        // (unless the launch has workgroups that do nothing else: sgd_reducers below)
        if (xstore && a.nred == 0) {
            int turn = 0;
            for (int pc = w; pc < npieces; pc += W, turn ^= 1) {
                long long *const red64 = reinterpret_cast<long long *>(L.red) + turn * (kWaves * kPiece);   // [kWaves][kPiece], two in turn
                const int sidx = pc * kPiece + (tid & (kPiece - 1));          // this thread's word
                const bool valid = sidx < NC * B || (side_step && sidx < nwords);
                long long sum = 0;
                if (valid) {
                    uint32_t spins = 0;
                    for (int row = tid / kPiece; row < W; row += kThreads / kPiece) {
                        const uint64_t *src = xpart + (size_t)row * xrow + sidx;
                        uint64_t v = load_dev(src);
#pragma unroll 1
                        while ((uint32_t)(v >> 48) != xtag && !dead) {
                            if (++spins > a.spin_limit) {
                                store_dev(a.status, (int)ZIPML_ETIMEOUT);
                                dead = true;
                            }
                            v = load_dev(src);
                        }
                        sum += tagged_value(v);
                    }
                }
                // lanes l, l + 8, ... of a wave hold the same word: add them, then the waves in LDS
                sum += __shfl_xor(sum, 8, kWave);
                sum += __shfl_xor(sum, 16, kWave);
                sum += __shfl_xor(sum, 32, kWave);
                if (lane < kPiece) red64[wave * kPiece + lane] = sum;
                lds_barrier();
                if (tid < kPiece) {
                    long long tot = 0;
#pragma unroll
                    for (int q = 0; q < kWaves; ++q) tot += red64[q * kPiece + tid];
                    if (valid) store_dev(xres + sidx, tag_word(xtag, tot));
                }
            }
        }

        ZIPML_TICK(3);
        // ============ residuals: poll the sums of this thread's samples
        float r[NC][kBpt];
        float rmax = 0.0f, rsum = 0.0f;
        if (xstore) {
            uint64_t raw[NC][kBpt], rawx = 0;
            const bool want_side = side_step && wave == 0;
            uint32_t spins = 0;
            if (tid < B || want_side) {
                const int watch = wave * kWave < B ? wave * kWave : 0;
#pragma unroll 1
                for (;;) {
                    // (one word first, as below)
                    if (!dead && (uint32_t)(load_dev(xres + watch) >> 48) != xtag) {
                        if (++spins > a.spin_limit) {
                            store_dev(a.status, (int)ZIPML_ETIMEOUT);
                            dead = true;
                        }
                        continue;
                    }
#pragma unroll
                    for (int cc = 0; cc < NC; ++cc)
#pragma unroll
                        for (int q = 0; q < kBpt; ++q) {
                            const int i = tid + q * nthr;
                            raw[cc][q] = load_dev(xres + cc * B + (i < B ? i : B - 1));
                        }
                    if (want_side) rawx = load_dev(xres + NC * B + (lane & 1));
                    bool all = !want_side || (uint32_t)(rawx >> 48) == xtag;
#pragma unroll
                    for (int cc = 0; cc < NC; ++cc)
#pragma unroll
                        for (int q = 0; q < kBpt; ++q) all = all && (uint32_t)(raw[cc][q] >> 48) == xtag;
                    if (all || dead) break;
                    if (++spins > a.spin_limit) {
                        store_dev(a.status, (int)ZIPML_ETIMEOUT);
                        dead = true;
                    }
                }
            }
            if (want_side && lane < 2) side[lane] = fixed_to_float(tagged_value(rawx), ky) * 1.00001f;
#pragma unroll
            for (int q = 0; q < kBpt; ++q) {
                const int i = tid + q * nthr;
#pragma unroll
                for (int cc = 0; cc < NC; ++cc) {
                    r[cc][q] = 0.0f;
                    if (i < B) {
                        r[cc][q] = fixed_to_float(tagged_value(raw[cc][q]), ky_pub) - bnext[q];
                        rmax = fmaxf(rmax, fabsf(r[cc][q]));
                        rsum += r[cc][q];
                    }
                }
                bnext[q] = bfut[q];
            }
        } else {
            uint64_t raw[NC][kBpt], rawx = 0;
            const bool want_side = side_step && wave == 0;     // wave 0 also fetches the side words
            uint32_t spins = 0;
            if (tid < B || want_side) {
                // A wave first watches ONE word (its first sample's: one request per round instead
                // of 64) and fetches the words of all its samples once that one is complete; the
                // workgroups contribute in the same order, so the others are then complete as
                // well, or are a round later.  With hundreds of workgroups polling, the requests
                // of the poll compete with the atomics they are waiting for.
                // (Only then: for a few workgroups the extra round trip costs more than it saves.)
                const int watch = wave * kWave < B ? wave * kWave : 0;
                const bool watch_first = (int64_t)W * B >= kWatchFirst;
#pragma unroll 1
                for (;;) {
                    if (watch_first && !dead && (int)(load_dev(acc + watch) >> kCountShift) != W) {
                        if (++spins > a.spin_limit) {
                            store_dev(a.status, (int)ZIPML_ETIMEOUT);
                            dead = true;
                        }
                        continue;
                    }
#pragma unroll
                    for (int cc = 0; cc < NC; ++cc)
#pragma unroll
                        for (int q = 0; q < kBpt; ++q) {
                            const int i = tid + q * nthr;
                            raw[cc][q] = load_dev(acc + cc * B + (i < B ? i : B - 1));
                        }
                    if (want_side) rawx = load_dev(acc + NC * B + (lane & 1));
                    bool all = !want_side || (int)(rawx >> kCountShift) == W;
#pragma unroll
                    for (int cc = 0; cc < NC; ++cc)
#pragma unroll
                        for (int q = 0; q < kBpt; ++q) all = all && (int)(raw[cc][q] >> kCountShift) == W;
                    if (all || dead) break;
                    if (++spins > a.spin_limit) {
                        store_dev(a.status, (int)ZIPML_ETIMEOUT);
                        dead = true;
                    }
                }
            }
            if (want_side && lane < 2) side[lane] = fixed_to_float(unpack_sum(rawx, W), ky_pub) * 1.00001f;
#pragma unroll
            for (int q = 0; q < kBpt; ++q) {
                const int i = tid + q * nthr;
#pragma unroll
                for (int cc = 0; cc < NC; ++cc) {
                    r[cc][q] = 0.0f;
                    if (i < B) {
                        r[cc][q] = fixed_to_float(unpack_sum(raw[cc][q], W), ky_pub) - bnext[q];
                        rmax = fmaxf(rmax, fabsf(r[cc][q]));
                        rsum += r[cc][q];
                    }
                }
                bnext[q] = bfut[q];
            }
        }
        if constexpr (kDbg) {
            if (a.dbg_r && blockIdx.x == 0) {     // intermediates of a production step (zipml_debug_step)
#pragma unroll
                for (int q = 0; q < kBpt; ++q) {
                    const int i = tid + q * nthr;
                    if (i < B) a.dbg_r[i] = r[0][q];
                }
            }
        }
        rmax = wave_reduce_dpp(rmax, [](float p, float q) { return fmaxf(p, q); });
        rsum = wave_sum_dpp(rsum);
        if (lane == 0) { wmax[wave] = rmax; wsum[wave] = rsum; }
        lds_barrier();
        ZIPML_TICK(4);

        // scale of the residuals, and the bounds for the next step's scale
        const float4 m0 = *reinterpret_cast<const float4 *>(wmax), m1 = *reinterpret_cast<const float4 *>(wmax + 4);
        const float4 s0 = *reinterpret_cast<const float4 *>(wsum), s1 = *reinterpret_cast<const float4 *>(wsum + 4);
        const float Rmax = fmaxf(fmaxf(fmaxf(m0.x, m0.y), fmaxf(m0.z, m0.w)), fmaxf(fmaxf(m1.x, m1.y), fmaxf(m1.z, m1.w)));
        const float Rtot = ((s0.x + s0.y) + (s0.z + s0.w)) + ((s1.x + s1.y) + (s1.z + s1.w));
        const int kr = Rmax < 3.0e38f ? scale_exponent(Rmax, 29) : 0;
        if (side_step) {
            beta_hat = side[0];
            ymax_hat = side[1] + ldexpf((float)W, -ky);     // |y_j| 2^ky <= |Y_j| + 1/2
        }
        rmax_step = fmaxf(rmax_step, Rmax);
        int ky_next = ky;
        if (last && !REP) {
            beta_hat += lr_abs * (lambda * rmax_step + l2_abs * beta_hat);
            ymax_hat += lr_abs * (mu * rmax_step + l2_abs * ymax_hat);
            ky_next = scale_of();
            rmax_step = 0.0f;
        }
        // residual digits
#pragma unroll
        for (int cc = 0; cc < NC; ++cc)
#pragma unroll
            for (int q = 0; q < kBpt; ++q) {
                const int i = tid + q * nthr;
                if (i < B)
                    store_digits(rdig + cc * NKS * 256 + r_pos[q],
                                 signed_digits(__float2int_rn(ldexpf(r[cc][q], kr))));
            }
        lds_barrier();
        ZIPML_TICK(8);
#ifdef ZIPML_STALE_DOT_EXPERIMENT
        // timing experiment: the next chunk's sums are published from the OLD model, before the
        // gradient pass (a one-step-delayed SGD; an upper bound on what a lookahead could gain)
        if (XM == 0 && NC == 1 && !REP && C == 1 && u + 1 < u_end) dot_and_publish(u + 1, ((t + 1) % kRefresh) == 0);
#endif

        // ============ gradient pass: one instruction per (16 features, 64 samples)
        {
            v4i c = {0, 0, 0, 0};
#pragma unroll
            for (int cc = 0; cc < NC; ++cc)
#pragma unroll
                for (int m = 0; m < kNG; ++m) {
                    const int ks = g_kh + KSS * m;
                    if (ks < NKS) {
                        v4i ad = {0, 0, 0, 0};
                        if (n16 < 4)
                            ad = *reinterpret_cast<const v4i *>(rdig + ((cc * NKS + ks) * 4 + n16) * 64 + q4 * 16);
                        c = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad, expand_codes<BITS>(c1[cc][m]), c, 0, 0, 0);
                    }
                }
#pragma unroll
            for (int m = 0; m < kNG; ++m) {
#pragma unroll
                for (int cc = 0; cc < NC; ++cc) p1ptr[cc][m] += step_dwords;
                if constexpr (kDouble) {
#pragma unroll
                    for (int k = 0; k < HW; ++k) c1[0][m][k] = c1nxt[m][k];
                }
            }
            if constexpr (!kDouble) {
                if (u + 1 < u_end) {
#pragma unroll
                    for (int cc = 0; cc < NC; ++cc) load_grad(cc, 0, c1[cc]);
                }
            }
            long long G = combine_digits(c);
            if (KSS > 1) {
                if (g_kh > 0 && lane < 16) gpart[g_kh * CW + oc] = G;
                lds_barrier();
                if (owner)
                    for (int kh = 1; kh < KSS; ++kh) G += gpart[kh * CW + oc];
            }
            ZIPML_TICK(9);
            // owners: gradient, update, next step's digits
            if (g_kh == 0) {
                if (owner) gsum += o_mid * Rtot + o_dl * fixed_to_float(G, kr);   // chunks in order
                if (last) {
                    int ky_own = ky_next;
                    if constexpr (REP) {
                        // ---- gradient exchange between the replicas of this feature block.  A
                        // 64-bit word carries, above the fp32 gradient share, a 16-bit tag of the
                        // step and an upper bound (8 significant bits) of the largest |residual|
                        // the replica saw, so one store delivers everything and its arrival.  Two
                        // buffers alternate (a workgroup cannot finish step t+1 before every
                        // replica has read step t: it needs their words of step t+1 first).
                        const size_t nfeat = (size_t)W * CW;
                        uint64_t *const gxb = a.gx + (size_t)(t & 1) * ((size_t)R * nfeat);
                        const uint32_t tag = ((uint32_t)(t + 1) & 0x7FFFu) | 0x8000u;
                        // bf16-like: truncate to 16 bits, one step up (rmax_step >= 0, finite or inf)
                        const uint32_t rbits = __float_as_uint(rmax_step);
                        const uint32_t r16 = rbits >= 0x7F800000u ? 0x7F80u : (rbits >> 16) + 1u;
                        if (owner)
                            store_dev(gxb + (size_t)rep * nfeat + j0 + oc,
                                      ((uint64_t)((tag << 16) | r16) << 32) | (uint64_t)__float_as_uint(gsum));
                        float gtot = 0.0f, rall = 0.0f;
                        if (owner) {
                            uint32_t spins = 0;
                            for (int q0 = 0; q0 < R; q0 += 8) {      // eight replicas per round of loads
                                uint64_t vg[8];
#pragma unroll 1
                                for (;;) {
                                    bool all = true;
#pragma unroll
                                    for (int q = 0; q < 8; ++q)
                                        if (q0 + q < R) {
                                            vg[q] = load_dev(gxb + (size_t)(q0 + q) * nfeat + j0 + oc);
                                            all = all && (uint32_t)(vg[q] >> 48) == tag;
                                        }
                                    if (all || dead) break;
                                    if (++spins > a.spin_limit) {
                                        store_dev(a.status, (int)ZIPML_ETIMEOUT);
                                        dead = true;
                                    }
                                }
#pragma unroll
                                for (int q = 0; q < 8; ++q)
                                    if (q0 + q < R) {                 // shares are added in replica order
                                        gtot += __uint_as_float((uint32_t)vg[q]);
                                        rall = fmaxf(rall, __uint_as_float(((uint32_t)(vg[q] >> 32) & 0xFFFFu) << 16));
                                    }
                            }
                        }
                        gsum = gtot;
                        if (g_ft == 0 && lane == 0) side[2] = rall;   // for everybody, after the next barrier
                        const float bh = beta_hat + lr_abs * (lambda * rall + l2_abs * beta_hat);
                        const float yh = ymax_hat + lr_abs * (mu * rall + l2_abs * ymax_hat);
                        const int k1 = scale_exponent(bh, 42), k2 = scale_exponent(yh, 29);
                        ky_own = k1 < k2 ? k1 : k2;                   // what scale_of() will give then
                    }
                    float xnew = 0.0f;
                    if (owner) {
                        const float g = o_live ? __fdiv_rn(gsum, (float)B * (float)(a.chunks * NC)) : 0.0f;
                        if constexpr (kDbg) {
                            if (a.dbg_g && o_live && rep == 0) a.dbg_g[j0 + oc] = g;
                        }
                        const float reg = a.l2 * x_own;
                        const float stp = a.lr * (g + reg);
                        x_own = x_own - stp;
                        if (a.prox) x_own = apply_prox(x_own, a.prox, a.lr, a.prox_coef);
                        xnew = x_own;
                    }
                    gsum = 0.0f;
#ifdef ZIPML_STALE_DOT_EXPERIMENT
                    refresh_y(xnew, ky_own, true);
#else
                    refresh_y(xnew, ky_own, side_next);
#endif
                }
            }
        }
        ky = ky_next;
        if (last) { chunk = 0; ++t; } else { ++chunk; }
        ZIPML_TICK(6);
    }
    if (owner) xs[oc] = x_own;
    lds_barrier();
#ifdef ZIPML_PHASE_TIMING
    if (w == 0 && tid == 0)
        for (int k = 0; k < 12; ++k) ((long long *)(a.nrm + 2048))[k] = prof_[k];
#endif
}

// Workgroups that only reduce (a.nred of them, behind the W workgroups that own features; plain
// estimator, no replicas): when a launch leaves compute units idle, they take the second trip of the
// exchange through tagged stores off the workgroups that own features -- whose polls of the rows
// otherwise queue behind their own loads of packed codes in the compute unit's memory pipeline, and
// which cannot start to reduce before their own dot pass is done.  Piece pc goes to reducer
// pc mod nred.  Same words, same tags, same buffers as in sgd_steps_mfma; a reducer leaves step u
// when it has stored its sums of step u, so it cannot run ahead of the owners (they need those
// sums), and every wait is bounded like theirs.
template <int UPT>
__device__ __forceinline__ void sgd_reducers(const SgdArgs &a, const Lds &L)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int W = a.W, B = a.B, FT = 2 * a.GQ;
    const int nw = (UPT == 1 && B <= 256 && FT <= 4) ? 4 : kWaves;
    if (nw != kWaves) return;                           // (the owners then exchange through atomics)
    const int rid = (int)blockIdx.x - W, nred = a.nred;
    const int C = a.chunks;
    const int64_t u_begin = a.step0 * C, u_end = (a.step0 + a.nsteps) * C;
    const int nwords = B + 2, xrow = a.xrow;
    // words per piece: eight, or four when there are reducers enough for pieces that small -- then
    // every thread polls one word of one row (128 rows of owners)
    const int piece = a.red_piece;
    const int npieces = (nwords + piece - 1) / piece;
    bool dead = false;
    int64_t t = a.step0;
    int chunk = 0;
    for (int64_t u = u_begin; u < u_end; ++u) {
        const bool side_step = chunk == 0 && (t % kRefresh) == 0;
        const uint32_t xtag = ((uint32_t)(u + 1) & 0x7FFFu) | 0x8000u;
        const uint64_t *const xpart = a.xpart + (size_t)(u & 1) * ((size_t)W * xrow);
        uint64_t *const xres = a.xpart + (size_t)2 * W * xrow + (size_t)(u & 1) * xrow;
        int turn = 0;
        for (int pc = rid; pc < npieces; pc += nred, turn ^= 1) {
            long long *const red64 = reinterpret_cast<long long *>(L.red) + turn * (kWaves * kPiece);   // (piece <= kPiece)
            const int sidx = pc * piece + (tid & (piece - 1));
            const bool valid = sidx < B || (side_step && sidx < nwords);
            // this thread's word in up to four rows (at most 256 owners, at least 64 threads per word):
            // all requested at once, and only those asked again that have not arrived
            long long sum = 0;
            if (valid) {
                const int stride = kThreads / piece;
                const uint64_t *src[4];
                uint64_t v[4];
                bool need[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int row = tid / piece + k * stride;
                    need[k] = row < W;
                    src[k] = xpart + (size_t)(need[k] ? row : 0) * xrow + sidx;
                    v[k] = need[k] ? load_dev(src[k]) : 0;
                }
                uint32_t spins = 0;
#pragma unroll 1
                while (!dead) {
                    bool all = true;
#pragma unroll
                    for (int k = 0; k < 4; ++k) all = all && (!need[k] || (uint32_t)(v[k] >> 48) == xtag);
                    if (all) break;
                    if (++spins > a.spin_limit) {
                        store_dev(a.status, (int)ZIPML_ETIMEOUT);
                        dead = true;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);        // (nothing else to do here: leave the memory side to the owners)
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (need[k] && (uint32_t)(v[k] >> 48) != xtag) v[k] = load_dev(src[k]);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (need[k]) sum += tagged_value(v[k]);
            }
            for (int sh = piece; sh < kWave; sh <<= 1) sum += __shfl_xor(sum, sh, kWave);
            if (lane < piece) red64[wave * piece + lane] = sum;
            lds_barrier();
            if (tid < piece) {
                long long tot = 0;
#pragma unroll
                for (int q = 0; q < kWaves; ++q) tot += red64[q * piece + tid];
                if (valid) store_dev(xres + sidx, tag_word(xtag, tot));
            }
        }
        if (chunk == C - 1) { chunk = 0; ++t; } else { ++chunk; }
    }
}

// Workgroups that only touch data (a.npref of them, behind the owners and the reducers; same
// launches as sgd_reducers): compute units that are still idle read the packed codes of the chunk
// two exchanges ahead, so that the owners find them in the cache in front of the memory instead
// of in the memory (the owners' loads sit in their compute unit's memory pipeline ahead of the
// polls of the exchange: with a data set small enough to stay in that cache the phases of a step
// add up to 0.4 us less).  The codes of chunk u are, for every group of 32 features and both
// copies, B * BITS consecutive dwords at (g n_pad + u B) BITS.  The segments are dealt out in
// turn; a prefetcher follows the exchange through the tag of the first result word (it reads the
// chunk c once the sums of chunk c - 2 exist, and leaves out the chunks it is late for) with a
// bounded wait, after which it stops waiting for good; it writes nothing.
template <int BITS>
__device__ __forceinline__ void sgd_prefetchers(const SgdArgs &a)
{
    const int tid = threadIdx.x;
    const int W = a.W, B = a.B;
    const int pid = (int)blockIdx.x - W - a.nred, np = a.npref;
    const int C = a.chunks;
    const int64_t u_begin = a.step0 * C, u_end = (a.step0 + a.nsteps) * C;
    const int xrow = a.xrow;
    const int64_t n_pad = a.nb64 * 64;
    const int nseg = 2 * a.d32;
    const int seg_bytes = B * BITS * 4;
    bool free_run = false;
    uint32_t sink = 0;
    // chunk c is read once the sums of chunk c - 2 exist; a prefetcher that finds the sums of chunk c
    // or of a later one there already is late and leaves chunk c out
    constexpr int kAhead = 2;            // (three and four chunks ahead were slower: 6.10 and 6.19 against 6.04 us per step)
    for (int64_t c = u_begin + kAhead; c < u_end; ++c) {
        if (!free_run) {
            const uint64_t *const word = a.xpart + (size_t)2 * W * xrow + (size_t)((c - kAhead) & 1) * xrow;   // result word 0 of chunks c - kAhead, + 2, ...
            const uint32_t want = (uint32_t)(c - kAhead + 1) & 0x7FFFu;
            uint32_t spins = 0;
            bool late = false;
#pragma unroll 1
            for (;;) {
                const uint32_t tag = (uint32_t)(load_dev(word) >> 48);
                // (never-written words have no tag bit; tags count chunks modulo 2^15)
                const uint32_t ahead = ((tag & 0x7FFFu) - want) & 0x7FFFu;
                if ((tag & 0x8000u) && ahead < 0x4000u) { late = ahead >= 2; break; }
                if (++spins > a.spin_limit) { free_run = true; break; }
                __builtin_amdgcn_s_sleep(4);
            }
            if (late) continue;
        }
        // eight segments' loads in flight per thread
        for (int off = tid * 16; off < seg_bytes; off += kThreads * 16) {
            for (int s0 = pid; s0 < nseg; s0 += 8 * np) {
                uint4 v[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int seg = s0 + k * np < nseg ? s0 + k * np : pid;
                    const int g = seg < a.d32 ? seg : seg - a.d32;
                    const unsigned char *base = reinterpret_cast<const unsigned char *>(seg < a.d32 ? a.p2 : a.p1) +
                                                ((size_t)g * (size_t)n_pad + (size_t)c * (size_t)B) * (size_t)(BITS * 4);
                    v[k] = *reinterpret_cast<const uint4 *>(base + off);
                }
#pragma unroll
                for (int k = 0; k < 8; ++k) sink ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
            }
        }
    }
    asm volatile("" ::"v"(sink));          // (the loads have a use; nothing is stored)
}

}  // namespace zipml
