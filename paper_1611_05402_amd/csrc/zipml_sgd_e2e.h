// Step loop of the epoch kernel in the end-to-end mode (Supp. C-E): the model is quantised before
// the dot pass (Q3), the mean gradient before the update (Q4), both with row scaling by the l2
// norm (Supp. A.3), so a step has three device-wide exchanges that depend on each other:
//     ||x||_2  ->  Q3, integer dot products  ->  residuals, gradient, ||g||_2  ->  Q4, update.
// Production launch only (persistent, more than one workgroup); included by zipml_sgd.hip and
// built on its SgdArgs / Lds / exchange-word helpers.  The stepwise and single-workgroup launches
// stay on sgd_steps<kInt>.
//
// Each exchange is ONE trip to the coherence point:
//   - the integer dot products travel like the fp32 ones (one 64-bit atomic per workgroup and
//     sample carrying arrival count and sum; every thread polls the words of its own samples);
//   - a norm is exchanged through one 64-bit slot per workgroup that holds the bits of the
//     workgroup's sum of squares PLUS ONE (sums are >= 0, so the bits never wrap; a zero slot means
//     "not there yet"): one store delivers value and arrival, and the waves that own features poll
//     all slots and add them up in registers.  The slots rotate over four buffers and are cleared
//     two steps ahead together with the dot-product words.
// The sums of squares are taken in fp64 in a fixed adjacent-pair tree over the feature index
// (inside a wave: butterfly over lanes, which is that tree because fp addition is commutative;
// then waves, then workgroups, pairwise), so the fp32 norm has the same bits on every workgroup
// and as a plain pairwise sum over the padded vector.
//
// Arithmetic per code: the dot pass adds T[j][code] = G[j][code] * m_j, a table rebuilt by the
// owner of feature j after Q3 (one LDS gather and one integer add per code; for wide level sets
// the product is formed on the fly); the gradient pass sums L[j][code] * r_i in fp64 (products of
// two fp32 numbers are exact there), so the mean gradient that Q4 quantises is the exact mean
// rounded to fp32, whatever the order.
#pragma once

namespace zipml {

// Sum over the 64 lanes in the adjacent-pair tree (lane order); every lane gets the result (fp
// addition is commutative, so the butterfly lane ^ 1, ^ 2, ... forms exactly that tree).  DPP row
// operations for the four levels inside a row of 16 lanes (after the two quad steps all lanes of
// a quad hold the quad's sum, so the mirror steps pair neighbouring quads and half rows), the
// cross-lane network for the rows.
template <int CTRL>
__device__ __forceinline__ double dpp_move_f64(double x)
{
    const long long b = __double_as_longlong(x);
    int blo = (int)(uint32_t)b, bhi = (int)(uint32_t)((uint64_t)b >> 32);
    asm volatile("" : "+v"(blo), "+v"(bhi));     // the source of a DPP move must sit in vector registers
    int lo = __builtin_amdgcn_update_dpp(0, blo, CTRL, 0xF, 0xF, true);
    int hi = __builtin_amdgcn_update_dpp(0, bhi, CTRL, 0xF, 0xF, true);
    asm volatile("" : "+v"(lo), "+v"(hi));       // (and the moves stay moves: no folding into the fp64 add)
    return __longlong_as_double((long long)(((uint64_t)(uint32_t)hi << 32) | (uint64_t)(uint32_t)lo));
}
__device__ __forceinline__ double wave_tree_sum_f64(double v)
{
    v = v + dpp_move_f64<0xB1>(v);     // lane ^ 1
    v = v + dpp_move_f64<0x4E>(v);     // lane ^ 2
    v = v + dpp_move_f64<0x141>(v);    // the other quad of the half row
    v = v + dpp_move_f64<0x140>(v);    // the other half row
    v = v + __shfl_xor(v, 16, kWave);  // the neighbouring row
    v = v + __shfl_xor(v, 32, kWave);  // the other pair of rows
    return v;
}

constexpr int kNormSlots = 256;   // slots per buffer of the norm exchange (>= workgroups)

template <int BITS, int UPT>
__device__ __forceinline__ void sgd_steps_e2e(const SgdArgs &a, const Lds &L)
{
    constexpr int K = 1 << BITS;
    constexpr bool kTable = BITS <= 4;               // T[j][c] = G[j][c] * m_j kept in LDS
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int w = blockIdx.x;
    const int W = a.W, GQ = a.GQ, CW = 32 * GQ, B = a.B;
    const int nrg = B >= 32 ? B / 32 : 1;
    const int j0 = w * CW;
    const int ngroups = (a.d32 - w * GQ) < GQ ? (a.d32 - w * GQ) : GQ;
    const float *Lg = a.levels + (size_t)j0 * K;
    float *const xs = L.xs, *const rs = L.rs;
    double *const red = L.red;
    double *const gpart = reinterpret_cast<double *>(L.gpart);
    int *const tq = L.tq;
    const bool is_owner = tid < CW;                  // this thread owns feature j0 + tid
    const int owner_waves = (CW + kWave - 1) / kWave;
    const bool owner_wave = wave < owner_waves;
    const int jme = j0 + tid;
    const bool live = is_owner && jme < a.d;
    const int s_m = (1 << (a.model_bits - 1)) - 1;
    const int s_g = a.grad_bits > 0 ? (1 << (a.grad_bits - 1)) - 1 : 1;
    const int nq = (W + kWave - 1) / kWave;          // norm slots per lane (W <= 256: at most 4)

    // ---- the units this thread owns, the same in every step (as in sgd_steps)
    int d_i[UPT], d_g[UPT];
#pragma unroll
    for (int k = 0; k < UPT; ++k) {
        int i = tid + k * kThreads, g = 0;
        while (i >= B && g < GQ) { i -= B; ++g; }
        d_i[k] = i;
        d_g[k] = g;
    }
    // all units of a thread belong to one sample (B == kThreads): their sums meet in a register
    bool one_sample = B == kThreads && ngroups <= UPT;
    const int nsl = kThreads / CW;
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
    auto load_labels = [&](int64_t t, float (&dst)[UPT]) {
#pragma unroll
        for (int k = 0; k < UPT; ++k) {
            const int i = tid + k * kThreads;
            if (i < B) dst[k] = a.b[t * B + i];
        }
    };

    bool dead = false;
    // One trip of the norm exchange.  sq: this thread's square (owners; 0 elsewhere), fp64.
    // Returns the l2 norm over all workgroups as fp32, to the owner waves (others get 0).
    auto exchange_norm = [&](double sq, uint64_t *slots) -> float {
        if (owner_wave) {
            sq = wave_tree_sum_f64(sq);
            if (lane == 0) red[wave] = sq;
        }
        lds_barrier();
        if (tid == 0) {
            double own = red[0];
            if (owner_waves == 2) own = red[0] + red[1];
            else if (owner_waves == 4) own = (red[0] + red[1]) + (red[2] + red[3]);
            store_dev(slots + w, (uint64_t)((uint64_t)__double_as_longlong(own) + 1ull));
        }
        if (!owner_wave) return 0.0f;
        uint64_t raw[4] = {1ull, 1ull, 1ull, 1ull};   // (bits of 0.0) + 1 for the slots past W
        uint32_t spins = 0;
#pragma unroll 1
        for (;;) {
            bool all = true;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q < nq && lane + kWave * q < W) {
                    raw[q] = load_dev(slots + lane + kWave * q);
                    all = all && raw[q] != 0ull;
                }
            if (__builtin_amdgcn_ballot_w64(!all) == 0ull || dead) break;
            if (++spins > a.spin_limit) {
                store_dev(a.status, (int)ZIPML_ETIMEOUT);
                dead = true;
            }
        }
        double s[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (q < nq) s[q] = wave_tree_sum_f64(__longlong_as_double((long long)(raw[q] - 1ull)));
        const double S = nq <= 1 ? s[0] : nq == 2 ? s[0] + s[1] : (s[0] + s[1]) + (s[2] + s[3]);
        return (float)sqrt(S);
    };

    const int64_t t_end = a.step0 + a.nsteps;
    uint32_t c2cur[UPT][BITS], c2nxt[UPT][BITS], c1cur[UPT][BITS], c1nxt[UPT][BITS];
    float bnext[UPT], bfut[UPT];
#pragma unroll
    for (int k = 0; k < UPT; ++k) bnext[k] = bfut[k] = 0.0f;
    load_dot_units(a.step0, c2cur);
    if (a.step0 + 1 < t_end) load_dot_units(a.step0 + 1, c2nxt);
    load_grad_units(a.step0, c1nxt);
    load_labels(a.step0, bnext);

    float x_own = is_owner ? xs[tid] : 0.0f;         // the owner keeps its weight in a register
    uint64_t *const slot_base = reinterpret_cast<uint64_t *>(a.nrm);

#ifdef ZIPML_PHASE_TIMING
    long long prof_[12] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    long long last_ = wall_clock64();
#endif
    for (int64_t t = a.step0; t < t_end; ++t) {
        uint64_t *const acc = a.acc + (size_t)(t & 3) * a.acc_words;
        uint64_t *const xn = slot_base + (size_t)(t & 3) * kNormSlots;
        uint64_t *const gn = slot_base + (size_t)(4 + (t & 3)) * kNormSlots;
        const int k0 = B >= 32 ? 0 : (int)((t * B) % 32);

        // ================= ||x||_2, Q3, the table of the dot pass
        const float Mx = exchange_norm(live ? (double)x_own * (double)x_own : 0.0, xn);
        ZIPML_TICK(0);
        const float sigma = Mx > 0.0f ? __fdiv_rn(Mx, (float)s_m) : 0.0f;
        if (owner_wave) {
            int mine = 0;
            if (live) {
                const Philox4 r = philox_block(a.seed, a.epoch, (uint64_t)t, (uint32_t)jme >> 2, 3u);
                mine = qvec_code(x_own, Mx, s_m, u24(philox_word(r, (uint32_t)jme & 3u)));
                if (a.dbg_m) a.dbg_m[jme] = mine;
            }
            if (is_owner) {
                L.ms[tid] = mine;
                if constexpr (kTable) {
#pragma unroll
                    for (int c = 0; c < K; ++c)
                        tq[tid * K + c] = (a.ident_grid ? c : (int)L.Gs[tid * K + c]) * mine;
                }
            }
            const int part = wave_sum_dpp(mine);
            if (lane == 0) L.isum[wave] = part;
            if (tid == 0) L.wsum[0] = sigma;          // for the threads outside the owner waves
        }
        lds_barrier();      // ms / tq / isum / sigma
        const float sigma_b = L.wsum[0];
        ZIPML_TICK(1);
        if (tid == 0) {
            int tot = 0;
            for (int q = 0; q < owner_waves; ++q) tot += L.isum[q];
            add_dev(acc + B, pack_int(tot));
        }

        // ================= dot pass: acc_i = sum_j G[j][c2_ij] m_j over the owned features
        {
            int pi[UPT];
#pragma unroll
            for (int k = 0; k < UPT; ++k) {
                pi[k] = 0;
                if (d_g[k] < ngroups) {
                    const int jb = d_g[k] * 32;
                    if constexpr (kTable) {
                        // (all lanes look up the same feature q at a time: K neighbouring words)
                        const int *T = tq + jb * K;
#pragma unroll
                        for (int q = 0; q < 32; ++q) {
                            pi[k] += T[q * K + (int)unit_code<BITS>(c2cur[k], q)];
                            if ((q & 15) == 15) asm volatile("" ::: "memory");   // sixteen look-ups in flight
                        }
                    } else {
                        pi[k] = unit_dot_int<BITS>(c2cur[k], a.ident_grid ? nullptr : L.Gs + jb * K, L.ms + jb, 0);
                    }
                }
            }
            if (one_sample) {
                int tot = 0;
#pragma unroll
                for (int k = 0; k < UPT; ++k) tot += pi[k];
                add_dev(acc + tid, pack_int(tot));
            } else if (ngroups > 1) {
#pragma unroll
                for (int k = 0; k < UPT; ++k)
                    if (d_g[k] < ngroups) L.zp[d_g[k] * B + d_i[k]] = (uint32_t)pi[k];
                lds_barrier();
                for (int i = tid; i < B; i += kThreads) {
                    int tot = 0;
                    for (int gq = 0; gq < ngroups; ++gq) tot += (int)L.zp[gq * B + i];
                    add_dev(acc + i, pack_int(tot));
                }
            } else {
#pragma unroll
                for (int k = 0; k < UPT; ++k)
                    if (d_g[k] < ngroups) add_dev(acc + d_i[k], pack_int(pi[k]));
            }
        }
        ZIPML_TICK(2);
        // The last wave of every workgroup clears its share of the exchange words, and its own norm
        // slots, of step t+2 (four buffers in rotation).  The workgroup is past the ||x|| exchange of
        // step t, so every workgroup has finished step t-1 and with it every read of step t-2, the
        // last user of these buffers; the stores are complete before this wave's poll below returns
        // (a wave's memory operations complete in order), hence before the workgroup contributes to
        // any later exchange, and nobody reaches step t+2 without those contributions.
        if (wave == kWaves - 1) {
            uint64_t *nxt = a.acc + (size_t)((t + 2) & 3) * a.acc_words;
            const int per = (B + 1 + W - 1) / W, hi = (w + 1) * per < B + 1 ? (w + 1) * per : B + 1;
            for (int i = w * per + lane; i < hi; i += kWave) store_dev(nxt + i, (uint64_t)0);
            if (lane == 0) {
                store_dev(slot_base + (size_t)((t + 2) & 3) * kNormSlots + w, (uint64_t)0);
                store_dev(slot_base + (size_t)(4 + ((t + 2) & 3)) * kNormSlots + w, (uint64_t)0);
            }
            if (!(tid < B)) vm_wait_all();
        }
        // rotate the register sets; request what later steps need right behind the atomics
#pragma unroll
        for (int k = 0; k < UPT; ++k)
#pragma unroll
            for (int q = 0; q < BITS; ++q) {
                c1cur[k][q] = c1nxt[k][q];
                c2cur[k][q] = c2nxt[k][q];
            }
        if (t + 1 < t_end) {
            load_grad_units(t + 1, c1nxt);
            load_labels(t + 1, bfut);
        }
        if (t + 2 < t_end) load_dot_units(t + 2, c2nxt);
        ZIPML_TICK(3);

        // ================= residuals: every thread polls the words of its own samples
        if (tid < B) {
            uint64_t raw[UPT], rawm = 0;
            uint32_t spins = 0;
#pragma unroll 1
            for (;;) {
#pragma unroll
                for (int q = 0; q < UPT; ++q) {
                    const int i = tid + q * kThreads;
                    raw[q] = load_dev(acc + (i < B ? i : B - 1));
                }
                rawm = load_dev(acc + B);
                bool all = (int)(rawm >> kCountShift) == W;
#pragma unroll
                for (int q = 0; q < UPT; ++q) all = all && (int)(raw[q] >> kCountShift) == W;
                if (all || dead) break;
                if (++spins > a.spin_limit) {
                    store_dev(a.status, (int)ZIPML_ETIMEOUT);
                    dead = true;
                }
            }
            const double summ = (double)unpack_sum(rawm, W);
#pragma unroll
            for (int q = 0; q < UPT; ++q) {
                const int i = tid + q * kThreads;
                if (i < B) {
                    const int av = (int)unpack_sum(raw[q], W);
                    const double z = (double)sigma_b * ((double)a.grid_lo * summ + (double)a.grid_step * (double)av);
                    const float r = (float)z - bnext[q];
                    rs[k0 + i] = r;
                    if (w == 0) {
                        if (a.dbg_acc) a.dbg_acc[i] = av;
                        if (a.dbg_r) a.dbg_r[i] = r;
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < UPT; ++q) bnext[q] = bfut[q];
        lds_barrier();    // rs[]
        ZIPML_TICK(4);

        // ================= gradient pass: fp64 sums over the samples of each owned unit
        {
            double part[UPT];
#pragma unroll
            for (int k = 0; k < UPT; ++k) {
                part[k] = 0.0;
                const int rgl = g_sl + k * nsl;
                if (g_live && rgl < nrg) {
                    // (rows of the LDS copy are K + 1 apart: lanes hold different features, and
                    // rows K apart would put all their look-ups on a few banks)
                    // (two loops: one pointer that may be LDS or global memory would be a generic one)
                    const float *rr = rs + rgl * 32;
                    double acc = 0.0;
                    if (a.lds_levels) {
                        const float *Lj = L.Lp + g_c * (K + 1);
#pragma unroll
                        for (int q = 0; q < 32; ++q) {
                            acc = fma((double)Lj[unit_code<BITS>(c1cur[k], q)], (double)rr[q], acc);
                            if ((q & 15) == 15) asm volatile("" ::: "memory");   // sixteen look-ups in flight
                        }
                    } else {
                        acc = unit_grad_table_f64<BITS>(c1cur[k], Lg + (size_t)g_c * K, rr);
                    }
                    part[k] = acc;
                }
            }
#pragma unroll
            for (int k = 0; k < UPT; ++k) {
                const int rgl = g_sl + k * nsl;
                if (rgl < nrg) gpart[rgl * CW + g_c] = part[k];
            }
        }
        lds_barrier();    // gpart[]
        ZIPML_TICK(5);
        float g = 0.0f;
        if (is_owner) {
            double sacc = 0.0;
            for (int r0 = 0; r0 < nrg; r0 += 8) {
                double v[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) v[q] = gpart[(r0 + q < nrg ? r0 + q : r0) * CW + tid];
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (r0 + q < nrg) sacc += v[q];
            }
            g = live ? (float)(sacc / (double)B) : 0.0f;      // the mean, rounded once
            if (a.dbg_g && live) a.dbg_g[jme] = g;
        }
        if (B < 32) {
            // a short batch shares its sample group with its neighbours: clear its residuals
            // (every read of rs[] is behind the barrier above; the next write is barriers away)
            for (int i = tid; i < B; i += kThreads) rs[k0 + i] = 0.0f;
        }

        ZIPML_TICK(6);
        // ================= ||g||_2, Q4, update
        if (a.grad_bits > 0) {
            const float Mg = exchange_norm(is_owner ? (double)g * (double)g : 0.0, gn);
            const float sg = Mg > 0.0f ? __fdiv_rn(Mg, (float)s_g) : 0.0f;
            if (live) {
                const Philox4 r = philox_block(a.seed, a.epoch, (uint64_t)t, (uint32_t)jme >> 2, 4u);
                const int code = qvec_code(g, Mg, s_g, u24(philox_word(r, (uint32_t)jme & 3u)));
                if (a.dbg_gq) a.dbg_gq[jme] = code;
                const float gh = sg * (float)code;
                const float stp = a.lr * gh;
                x_own = x_own - stp;
            }
        } else if (live) {
            const float stp = a.lr * g;
            x_own = x_own - stp;
        }
        ZIPML_TICK(7);
    }
    if (is_owner) xs[tid] = x_own;
    lds_barrier();
#ifdef ZIPML_PHASE_TIMING
    if (w == 0 && tid == 0)
        for (int k = 0; k < 12; ++k) ((long long *)(a.nrm + 2048))[k] = prof_[k];
#endif
}

}  // namespace zipml
