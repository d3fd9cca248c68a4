// Epoch kernel for very large minibatches: workgroups own samples, not features (included by
// zipml_sgd.hip after zipml_sgd_mfma.h, whose operand helpers it uses).
//
// Same estimator, eq. (5) of Sec. 2.2, g = mean_i Q1(a_i) (Q2(a_i)^T x - b_i), evenly spaced
// levels, fp32 model, 2-, 4- or 8-bit codes.  When a minibatch has many more samples than the
// device has lanes, the exchange of per-sample partial sums between feature owners (one atomic
// per workgroup and sample) is what bounds the feature-owner kernel; here a workgroup takes
// whole samples instead: tiles of 64 samples times all features.  It keeps the digits of
// y_j = delta_j x_j of the whole model in LDS, so the dot products of its samples are complete
// inside the workgroup, forms their residuals at once and runs the gradient pass over the same 64
// samples straight away, adding into a gradient of all features that it keeps in LDS.  Per step
// the workgroups meet twice: after their tiles, to add up the per-workgroup gradients (each wave
// sums 16 features over all workgroups, in a fixed order) and update the model in place; and after
// that update.  Nothing else is exchanged, so the packed data streams at the rate the memory
// system delivers it: every wave keeps one item (16 to 32 packed dwords per lane, requested with
// non-temporal loads that no branch can skip) in flight while it feeds the previous one to the
// matrix cores.
//
// The symmetrised estimator (Supp. B.2, footnote; AVG) runs every tile of samples twice, once per code pair
// -- (copy 2, copy 1) and (copy 1 sample-major, copy 2 feature-major) -- into the same gradient,
// which is then the sum over both pairs, and the sum of residuals the sum over both.
//
// Arithmetic is that of the matrix-core step loop: y and the residuals of a tile as 32-bit fixed
// point in four signed base-256 digits, v_mfma_i32_16x16x64_i8 against the codes expanded to
// bytes, exact integer sums, one rounding back to fp32 per tile and feature.  The fixed-point
// scales are taken from the data themselves (max_j |y_j| once per step, max_i |r_i| per tile).
#pragma once

namespace zipml {

struct RowsArgs {
    const uint32_t *p1, *p2;
    const uint32_t *p1s, *p2s;   // symmetrised estimator: copy 2 feature-major, copy 1 sample-major
    const float *b;
    float *x;
    const float *dl, *mid;   // [NKB * 64] delta_j and lo_j + off * delta_j (zero beyond d), from k_sgd_prepare
    int64_t n_pad, n32;      // samples per feature group of copy 2, sample groups of copy 1
    int d, d32, NKB;         // features, feature groups, 64-feature blocks
    int64_t B;               // minibatch (multiple of 64)
    int64_t step0;
    int nsteps;
    float lr, l2;
    int prox;                // proximal step after the update (ZIPML_PROX_*)
    float prox_coef;
    int *status;
    uint32_t *sync;
    const int *even;         // [kEvenBlocks] from k_sgd_prepare
    float *part;             // [gridDim.x][NKB * 64] per-workgroup gradients, then [gridDim.x] sums of residuals
    uint32_t spin_limit;
};

// KPI: 64-feature blocks per wave and item (at most 16 / BITS: 32 packed dwords per lane in flight
// per item; less when the problem has fewer than 8 * KPI blocks).
template <int BITS, int KPI, bool AVG>
__device__ __forceinline__ void sgd_rows(const RowsArgs &a, unsigned char *smem)
{
    constexpr int HW = BITS / 2;          // packed dwords per lane operand (16 codes)
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // the same for the whole wave: scalar addresses
    const int n16 = lane & 15, q4 = lane >> 4;
    const int P = gridDim.x, p = blockIdx.x;
    const int NKB = a.NKB, nfeat = NKB * 64;
    const int NG = (NKB + kWaves * KPI - 1) / (kWaves * KPI);   // items per pass and tile
    // tiles of a minibatch; with two code pairs tile V is samples 64 (V / 2) .. of pair V % 2
    constexpr int PS = AVG ? 1 : 0;
    const int64_t NT = (a.B / 64) << PS;

    // ---- LDS
    int8_t *const ydig = (int8_t *)smem;                               // [NKB][4 digits][4 q][16]
    float *const gs = (float *)(smem + (size_t)NKB * 256);             // [NKB * 64] gradient of this workgroup
    unsigned char *tail = smem + (size_t)NKB * 512;
    long long *const zpart = (long long *)tail;                        // [kWaves][64] partial dot products
    int8_t *const rdig = (int8_t *)(tail + kWaves * 64 * 8);           // [4 digits][4 q][16]
    float *const red = (float *)(tail + kWaves * 64 * 8 + 256);        // [2 * kWaves] block reductions
    int *const misc = (int *)(tail + kWaves * 64 * 8 + 256 + 64);      // [0] kr of the tile
    int8_t *const zeros = (int8_t *)(tail + kWaves * 64 * 8 + 256 + 128);   // [16] zero bytes
    if (tid < 4) reinterpret_cast<int *>(zeros)[tid] = 0;

    // evenly spaced levels everywhere?  (found by the preparation kernel)
    {
        int ok_all = 1;
        if (tid < Workspace::kEvenBlocks) ok_all = a.even[tid];
        if (!__syncthreads_and(ok_all)) {
            if (p == 0 && tid == 0) store_dev(a.status, (int)ZIPML_EUNSUPPORTED);
            return;
        }
    }

    uint32_t passed = 0;
    bool dead = false;
    auto grid_sync = [&]() {
        vm_wait_all();            // this wave's device-scope stores have been acknowledged
        __syncthreads();
        if (tid == 0) {
            ++passed;
            add_dev(a.sync, 1u);
            const uint32_t target = passed * (uint32_t)P;
            uint32_t spins = 0;
#pragma unroll 1
            while (!dead && load_dev(a.sync) < target) {
                if (++spins > a.spin_limit) {
                    store_dev(a.status, (int)ZIPML_ETIMEOUT);
                    dead = true;
                }
            }
        }
        __syncthreads();
    };

    // where the digits of feature / sample e (inside its block of 64) go: the operand map of code_slot
    auto digit_pos = [](int e) {
        int half, byte;
        code_slot<BITS>(e & 31, half, byte);
        return (2 * ((e >> 5) & 1) + half) * 16 + byte;
    };
    const int my_pos = digit_pos(lane);
    // Four 16-sample (16-feature) tiles share one accumulator: the digit operand of tile slot sl
    // has the digits in rows 4 sl .. 4 sl + 3 and zeros elsewhere, so the sums of slot sl land in
    // lanes 16 sl .. 16 sl + 15.  A lane reads its 16 operand bytes either from the digits or from
    // 16 zero bytes: dig_off is its offset inside a block of digits, and slot_of its slot.
    const int dig_off = (n16 & 3) * 64 + q4 * 16, slot_of = n16 >> 2;
    const int zero_off = (int)(zeros - ydig);

    // ---- packed data in flight: two items of KPI x 4 lane operands
    uint32_t buf0[KPI][4][HW], buf1[KPI][4][HW];
    // item k of a tile: k < NG dot pass (copy 2), else gradient pass (copy 1); block index of slot j
    auto block_of = [&](int k, int j) { return wave + kWaves * (KPI * (k < NG ? k : k - NG) + j); };
    // An address is a base that is the same for the whole wave (scalar registers) plus a small
    // per-lane byte offset:
    //   copy 2: lane = sample 16 sl + n16 of the tile, 16 codes (half q4 & 1) of feature group 2 kb + q4 / 2
    //   copy 1: lane = feature 64 kb + 16 sl + n16, 16 codes (half q4 & 1) of sample group row0 / 32 + q4 / 2
    // A 64-feature block whose second group is padding (odd number of groups) reads its first
    // group twice; the digits of y there are zero, and its gradient is never used.
    const uint32_t dot_lo = (uint32_t)((n16 * BITS + (q4 & 1) * HW) * 4);
    const uint32_t dot_hi = (uint32_t)((q4 >> 1) * a.n_pad * BITS * 4);
    const uint32_t grad_off = (uint32_t)((((q4 >> 1) * 32 + n16) * BITS + (q4 & 1) * HW) * 4);
    // (Choices between the two passes are written as masks, not as selections between variables:
    // a selection between two captured variables would keep them, and everything around them,
    // in memory.)
    const uintptr_t copy1 = (uintptr_t)a.p1, copy_diff = (uintptr_t)a.p2 - (uintptr_t)a.p1;
    // (second code pair: what the first copy moves by, and what the difference between the copies moves by)
    const uintptr_t pair_diff = AVG ? (uintptr_t)a.p1s - (uintptr_t)a.p1 : 0;
    const uintptr_t pair_copy_diff = AVG ? ((uintptr_t)a.p2s - (uintptr_t)a.p1s) - copy_diff : 0;
    const uint32_t off_diff = dot_lo - grad_off;
    const int d32 = a.d32;
    // In both copies a 64-feature block is 8 * BITS * n_pad bytes from the next, and the 64 samples
    // of a tile start 4 * BITS * row0 bytes into a feature group (copy 1: n32 * 32 = n_pad samples
    // per group, 32 * BITS dwords per sample group).  So an address is
    //   copy + 4 BITS row0 + kb * block_bytes + (a few hundred bytes that depend on sl) + lane offset,
    // and only the first three terms need 64-bit arithmetic, once per block.
    const uintptr_t block_bytes = (uintptr_t)8 * BITS * (uintptr_t)a.n_pad;
    // Every call requests the same number of loads, whatever the item, and no load sits behind a
    // branch: only then can the wait for an item leave exactly the next item's loads in flight.
    // (Blocks past the last one repeat it; nothing is computed from them.)
    auto issue = [&](int64_t row0, int pair, int k, uint32_t (&dst)[KPI][4][HW]) __attribute__((always_inline)) {
        const uintptr_t dm = (uintptr_t)0 - (uintptr_t)(k < NG ? 1 : 0);   // all ones: dot pass
        uintptr_t tile = copy1 + (copy_diff & dm) + (uintptr_t)(4 * BITS) * (uintptr_t)row0;
        if constexpr (AVG) {
            const uintptr_t pm = (uintptr_t)0 - (uintptr_t)pair;            // all ones: second pair
            tile += (pair_diff & pm) + (pair_copy_diff & pm & dm);
        }
        const int kb0 = wave + kWaves * KPI * (k < NG ? k : k - NG);
#pragma unroll
        for (int j = 0; j < KPI; ++j) {
            int kb = kb0 + kWaves * j;
            kb = kb < NKB ? kb : NKB - 1;
            const uint32_t whole = 2 * kb + 1 < d32 ? ~0u : 0u;
            const uintptr_t block = tile + (uintptr_t)kb * block_bytes;
            const uint32_t off = grad_off + ((off_diff + (dot_hi & whole)) & (uint32_t)dm);
            // second feature group of the block (copy 1, sl >= 2): half a block further
            const uintptr_t second = (block_bytes >> 1) & (uintptr_t)(int64_t)(int32_t)whole;
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                const uintptr_t in_dot = (uintptr_t)(64 * BITS * sl);
                const uintptr_t in_grad = (sl >> 1 ? second : 0) + (uintptr_t)(64 * BITS * (sl & 1));
                const uintptr_t base = block + in_grad + ((in_dot - in_grad) & dm);
                // (a pointer rebuilt from an integer: say that it points to global memory; the
                // vector type carries the alignment)
                typedef uint32_t words_t __attribute__((ext_vector_type(HW)));
                // (non-temporal: every packed byte is read once per step; letting the stream allocate
                // in the L2 as ordinary loads do cost 12-16 % of the rate)
                const words_t v = __builtin_nontemporal_load((const __attribute__((address_space(1))) words_t *)(base + off));
#pragma unroll
                for (int h = 0; h < HW; ++h) dst[j][sl][h] = HW == 1 ? ((const uint32_t *)&v)[0] : v[h];
            }
        }
    };

    const int64_t t_end = a.step0 + a.nsteps;
    // The packed data do not depend on the model: the first item of a step is requested before the
    // previous step's gradients are added up (here: before the first step's model is read).
    if (p < NT) issue(a.step0 * a.B + 64 * (int64_t)(p >> PS), p & PS, 0, buf0);
#ifdef ZIPML_PHASE_TIMING
    long long prof_[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = wall_clock64();
#define ZIPML_RTICK(k) do { if (p == 0 && tid == 0) { const long long now_ = wall_clock64(); prof_[k] += now_ - last_; last_ = now_; } } while (0)
#else
#define ZIPML_RTICK(k) do { } while (0)
#endif
    for (int64_t t = a.step0; t < t_end; ++t) {
        ZIPML_RTICK(5);
        // ============ the model of this step: digits of y_j = delta_j x_j, sum_j mid_j x_j
        // (the model was written by other workgroups: device-scope loads, four in flight per thread;
        // y_j waits in the gradient array until the scale is known)
        float ymax = 0.0f, cqp = 0.0f;
        for (int j0 = 0; j0 < nfeat; j0 += 4 * kThreads) {
            float xv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = j0 + tid + e * kThreads;
                xv[e] = j < a.d ? load_dev(a.x + j) : 0.0f;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = j0 + tid + e * kThreads;
                if (j < nfeat) {
                    const float y = a.dl[j] * xv[e];
                    ymax = fmaxf(ymax, fabsf(y));
                    cqp += a.mid[j] * xv[e];
                    gs[j] = y;
                }
            }
        }
        ymax = wave_reduce_dpp(ymax, [](float u, float v) { return fmaxf(u, v); });
        cqp = wave_sum_dpp(cqp);
        __syncthreads();                       // everybody is done with the previous step's LDS
        if (lane == 0) { red[wave] = ymax; red[kWaves + wave] = cqp; }
        __syncthreads();
        float cq = 0.0f;
        ymax = 0.0f;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) { ymax = fmaxf(ymax, red[v]); cq += red[kWaves + v]; }
        const int ky = scale_exponent(ymax, 29);
        for (int j = tid; j < nfeat; j += kThreads) {
            const int Y = __float2int_rn(ldexpf(gs[j], ky));
            store_digits(ydig + (j >> 6) * 256 + digit_pos(j & 63), signed_digits(Y));
            gs[j] = 0.0f;
        }
        float rtot = 0.0f;                     // wave 0: sum of this workgroup's residuals
        __syncthreads();
        ZIPML_RTICK(0);

        // ============ tiles of 64 samples: dot pass, residuals, gradient pass.  The tiles are
        // dealt out in turn (tile T to workgroup T mod P).  Handing them out by a counter instead
        // was tried: it costs an atomic per tile, makes the order of the fp32 sums -- and with it
        // the last bits of the result -- depend on timing, and gained nothing: the workgroups
        // finish within one tile of each other either way.
        for (int64_t T = p; T < NT; T += P) {
            const int64_t row0 = t * a.B + 64 * (T >> PS);
            const int pair = (int)(T & PS);
            const float label = a.b[row0 + lane];      // (every wave: no load behind a branch)
            v4i cdot = {0, 0, 0, 0};
            // one item: request the next one, then feed this one to the matrix cores
            auto item = [&](int k, uint32_t (&cur)[KPI][4][HW], uint32_t (&nxt)[KPI][4][HW]) __attribute__((always_inline)) {
                // (after the last tile of a step: the first tile of the next step; after the last
                // step: this tile's first item again, never used)
                const bool more = k + 1 < 2 * NG;
                if constexpr (AVG) {
                    const int64_t t_next = T + P < NT ? t : t + 1 < t_end ? t + 1 : t;
                    const int64_t T_next = T + P < NT ? T + P : t + 1 < t_end ? (int64_t)p : T;
                    const int64_t row_next = t_next * a.B + 64 * (T_next >> 1);
                    issue(more ? row0 : row_next, more ? pair : (int)(T_next & 1), more ? k + 1 : 0, nxt);
                } else {
                    const int64_t row_next = T + P < NT ? row0 + 64 * (int64_t)P
                                             : t + 1 < t_end ? (t + 1) * a.B + 64 * (int64_t)p : row0;
                    issue(more ? row0 : row_next, 0, more ? k + 1 : 0, nxt);
                }
                if (k == NG) {
                    // ---- residuals of the tile (wave 0), between the two passes
                    zpart[wave * 64 + lane] = combine_digits(cdot);
                    lds_barrier();          // (not __syncthreads: that would also wait for the loads in flight)
                    if (wave == 0) {
                        long long z = 0;
#pragma unroll
                        for (int v = 0; v < kWaves; ++v) z += zpart[v * 64 + lane];
                        const float r = (float)(ldexp((double)z, -ky) + (double)cq) - label;
                        const float rmax = wave_reduce_dpp(fabsf(r), [](float u, float v) { return fmaxf(u, v); });
                        rtot += wave_sum_dpp(r);
                        const int kr = rmax < 3.0e38f ? scale_exponent(rmax, 29) : 0;
                        store_digits(rdig + my_pos, signed_digits(__float2int_rn(ldexpf(r, kr))));
                        if (lane == 0) misc[0] = kr;
                    }
                    lds_barrier();
                }
                if (k < NG) {
#pragma unroll
                    for (int j = 0; j < KPI; ++j) {
                        const int kb = block_of(k, j);
                        if (kb < NKB) {
#pragma unroll
                            for (int sl = 0; sl < 4; ++sl) {
                                const v4i ad = *reinterpret_cast<const v4i *>(
                                    ydig + (slot_of == sl ? kb * 256 + dig_off : zero_off));
                                cdot = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad, expand_codes<BITS>(cur[j][sl]),
                                                                             cdot, 0, 0, 0);
                            }
                        }
                    }
                } else {
                    const int kr = misc[0];
                    const int rdig_off = (int)(rdig - ydig);
#pragma unroll
                    for (int j = 0; j < KPI; ++j) {
                        const int kb = block_of(k, j);
                        if (kb < NKB) {
                            v4i c = {0, 0, 0, 0};
#pragma unroll
                            for (int sl = 0; sl < 4; ++sl) {
                                const v4i ad = *reinterpret_cast<const v4i *>(
                                    ydig + (slot_of == sl ? rdig_off + dig_off : zero_off));
                                c = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad, expand_codes<BITS>(cur[j][sl]), c, 0, 0, 0);
                            }
                            // lane = feature 64 kb + lane: its four digits sit in this lane
                            gs[kb * 64 + lane] += fixed_to_float(combine_digits(c), kr);
                        }
                    }
                }
            };
            for (int k = 0; k < 2 * NG; k += 2) {
                item(k, buf0, buf1);
                item(k + 1, buf1, buf0);
            }
        }

        // ============ gradients of all workgroups -> model
        ZIPML_RTICK(1);
        __syncthreads();
        float *const mine = a.part + (size_t)p * nfeat;
        for (int j = tid; j < nfeat; j += kThreads) store_dev(mine + j, gs[j]);
        if (tid == 0) store_dev(a.part + (size_t)P * nfeat + p, rtot);
        grid_sync();
        ZIPML_RTICK(2);
        {
            // A wave sums 16 features over all workgroups: lane (n16, q4) takes workgroups q4,
            // q4 + 4, ...  Everything it needs -- up to 64 partial gradients per lane, its share of
            // the sums of residuals, the model -- is requested in one go; all sums are taken in a
            // fixed order.
            const int nblk = nfeat / 16;
            const float *const rsum_all = a.part + (size_t)P * nfeat;
            for (int jb = p * kWaves + wave; jb < nblk; jb += P * kWaves) {
                const int j = jb * 16 + n16;
                const float xj = load_dev(a.x + (j < a.d ? j : 0));
                float rv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int q = lane + e * kWave;
                    rv[e] = load_dev(rsum_all + (q < P ? q : P - 1));
                    rv[e] = q < P ? rv[e] : 0.0f;
                }
                float s = 0.0f;
                for (int q0 = q4; q0 < P; q0 += 256) {      // (one round for up to 256 workgroups)
                    float v[64];
#pragma unroll
                    for (int e = 0; e < 64; ++e) {
                        const int q = q0 + 4 * e;
                        v[e] = load_dev(a.part + (size_t)(q < P ? q : P - 1) * nfeat + j);
                    }
#pragma unroll
                    for (int e = 0; e < 64; ++e) s += q0 + 4 * e < P ? v[e] : 0.0f;
                }
                float rs = (rv[0] + rv[1]) + (rv[2] + rv[3]);
                for (int q = lane + 4 * kWave; q < P; q += kWave) rs += load_dev(rsum_all + q);   // (more than 256 workgroups)
                const float Rtot = wave_sum_dpp(rs);
                const float s0 = __shfl(s, n16, kWave), s1 = __shfl(s, 16 + n16, kWave);
                const float s2 = __shfl(s, 32 + n16, kWave), s3 = __shfl(s, 48 + n16, kWave);
                const float G = (s0 + s1) + (s2 + s3);
                if (q4 == 0 && j < a.d) {
                    // (two code pairs: both sums run over twice the samples, and the estimator is their mean)
                    const float g = __fdiv_rn(a.mid[j] * Rtot + a.dl[j] * G, (float)(a.B << PS));
                    const float reg = a.l2 * xj;
                    const float stp = a.lr * (g + reg);
                    const float v = xj - stp;
                    store_dev(a.x + j, a.prox ? apply_prox(v, a.prox, a.lr, a.prox_coef) : v);
                }
            }
        }
        ZIPML_RTICK(3);
        if (t + 1 < t_end) grid_sync();      // (after the last step the end of the kernel is the meeting)
        ZIPML_RTICK(4);
    }
#ifdef ZIPML_PHASE_TIMING
    if (p == 0 && tid == 0)
        for (int k = 0; k < 8; ++k) ((long long *)(a.part + (size_t)P * nfeat + P))[k] = prof_[k];   // spare words behind the sums
#endif
}

template <int BITS, int KPI, bool AVG = false>
__global__ __launch_bounds__(kThreads, 1) void k_sgd_rows(RowsArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    sgd_rows<BITS, KPI, AVG>(a, smem);
}

// LDS of k_sgd_rows for NKB blocks of 64 features.
__host__ __device__ inline size_t rows_lds_bytes(int NKB)
{
    return (size_t)NKB * 512 + kWaves * 64 * 8 + 256 + 64 + 64 + 16;
}

}  // namespace zipml
