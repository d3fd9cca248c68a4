// The sample-owner epoch kernel for 2-bit codes with the dot pass on the 4-bit floating-point
// matrix instruction (included by zipml_sgd.hip after zipml_sgd_rows.h, whose arguments, reduction
// and host helpers it shares).
//
// Same estimator and the same integer dot products and gradient sums as k_sgd_rows<2, ...> (eq. (5),
// Sec. 2.2; with tiles of 64 samples the model after an epoch is bit-identical, with larger tiles
// the fp32 sums over tiles and workgroups run in another order).  What differs is how the dot pass feeds the matrix cores.  At 2 bits
// k_sgd_rows is bound by instruction issue, not by memory: per 16 codes a lane spends seven vector
// instructions on turning them into bytes and one v_mfma_i32_16x16x64_i8 of which 4 of 16 rows
// carry digits -- four times the instructions per packed byte of the 8-bit kernel (counters: 46 %
// of the busy cycles vector ALU, 47 % matrix cores, 49 % of the HBM peak).
// v_mfma_f32_16x16x128_f8f6f4 with both operands in E2M1 takes 32 values a lane and is twice as deep:
//   - a 2-bit code c, left in the low bits of a nibble, IS the E2M1 number c / 2 (0, 0.5, 1, 1.5), so
//     a packed dword becomes two operand dwords with three instructions (p & 0x33333333,
//     (p >> 2) & 0x33333333: even codes, then odd codes; the digits are laid out to match);
//   - y_j 2^ky, a 30-bit integer, is written in base 4 with digits -2 .. 1 (add 2 to every digit,
//     take the bits, subtract again), all of them E2M1 numbers: 15 signed digits and a 16th that is
//     0 or 1 fill the 16 rows of the other operand, none idle;
//   - products and sums are small half-integers, exact in fp32; a lane folds its four rows with
//     three multiply-adds and the rest of the digit sum is integer arithmetic in LDS, once per tile.
// One matrix instruction and six vector instructions per 32 codes instead of two and fourteen.
// The gradient pass stays on v_mfma_i32_16x16x64_i8 as in k_sgd_rows: its result is a different
// feature for every instruction, and folding sixteen digit rows across four lane groups per
// instruction would cost what the operand conversion saves.
//
// Operand layout of the instruction (checked on the device against a host product of random E2M1
// values and with one-hot operands): A: lane l holds row l % 16, k = 32 (l / 16) .. + 31, nibble j of
// its 128 bits is k = 32 (l / 16) + j; B the same with columns; C: lane l holds column l % 16,
// rows 4 (l / 16) .. + 3.
#pragma once

namespace zipml {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

// LDS of k_sgd_rows_fp4 for NKB blocks of 64 features: digits of y (1 KiB per 128 features), the
// workgroup's gradient, then per wave and sample the four folded row groups, residual digits, ...
// (TM: a tile is 64 TM samples)
__host__ __device__ inline size_t rows_fp4_lds_bytes(int NKB, int TM)
{
    return (size_t)((NKB + 1) / 2) * 1024 + (size_t)NKB * 256 + (size_t)TM * (kWaves * 64 * 16 + 256) + 64 + 64 + 16;
}

// TM: sample blocks of 64 per tile.  What a tile costs beside its data -- two workgroup barriers,
// the residuals in one wave between them, the pipeline of requests running empty and filling again
// -- does not depend on the code width, and at 2 bits a tile of 64 samples is only a quarter of the
// data of an 8-bit tile: with 64-sample tiles this kernel stayed at 45 % of the HBM peak even with
// its matrix instructions taken out.  Larger tiles also let the gradient pass add TM times as many
// matrix instructions into an accumulator before it folds the digits.
template <int TM>
__device__ __forceinline__ void sgd_rows_fp4(const RowsArgs &a, unsigned char *smem)
{
    constexpr int BITS = 2, TS = 64 * TM, NSL = 4 * TM, NW = 8 * TM;   // samples, 16-sample slots, dwords of an item
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n16 = lane & 15, q4 = lane >> 4;
    const int P = gridDim.x, p = blockIdx.x;
    const int NKB = a.NKB, nfeat = NKB * 64;
    const int NB = (NKB + 1) / 2;                       // blocks of 128 features
    const int ND = (NB + kWaves - 1) / kWaves;          // blocks per wave: items per pass and tile
    const int64_t NT = a.B / TS;

    // ---- LDS
    unsigned char *const ydig = smem;                                   // [NB][16 rows][4 q][16 bytes of nibbles]
    float *const gs = (float *)(smem + (size_t)NB * 1024);              // [NKB * 64] gradient of this workgroup
    unsigned char *tail = smem + (size_t)NB * 1024 + (size_t)NKB * 256;
    int *const zq = (int *)tail;                                        // [kWaves][TS samples][4 row groups]
    int8_t *const rdig = (int8_t *)(tail + TM * kWaves * 64 * 16);      // [TM][4 digits][4 q][16]
    unsigned char *const tail2 = tail + TM * (kWaves * 64 * 16 + 256);
    float *const red = (float *)tail2;                                  // [2 * kWaves]
    int *const misc = (int *)(tail2 + 64);                              // [0] kr of the tile
    int8_t *const zeros = (int8_t *)(tail2 + 128);                      // [16] zero bytes
    if (tid < 4) reinterpret_cast<int *>(zeros)[tid] = 0;

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
        vm_wait_all();
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

    // residual digits (gradient pass, as k_sgd_rows<2>): the operand map of code_slot
    int my_pos;
    {
        int half, byte;
        code_slot<BITS>(lane & 31, half, byte);
        my_pos = (2 * ((lane >> 5) & 1) + half) * 16 + byte;
    }
    const int dig_off = (n16 & 3) * 64 + q4 * 16, slot_of = n16 >> 2;

    // ---- packed data in flight: one item of 8 TM dwords while the one before is computed on.  A dot item is one 128-feature block
    // of copy 2 (lane = sample 16 sl + n16 of the tile, the 32 codes of feature group 4 KB + q4:
    // one packed unit, two dwords); a gradient item is the same block of copy 1 (its two halves of
    // 64 features: lane = feature 64 kb + 16 sl + n16, 16 codes -- half q4 & 1 -- of sample group
    // row0 / 32 + q4 / 2: one dword).  Groups past the last one repeat it: their digits are zero,
    // their gradients unused.
    uint32_t buf0[NW], buf1[NW];
    const uintptr_t copy1 = (uintptr_t)a.p1, copy2 = (uintptr_t)a.p2;
    const int d32 = a.d32;
    const int64_t n_pad = a.n_pad, n32 = a.n32;
    typedef uint32_t pair_t __attribute__((ext_vector_type(2)));
    // item s of a tile: s < ND dot pass, else gradient pass; block of item s: wave + kWaves * (s mod ND)
    auto issue = [&](int64_t row0, int s, uint32_t (&dst)[NW]) __attribute__((always_inline)) {
        const bool dot = s < ND;
        int KB = wave + kWaves * (dot ? s : s - ND);
        KB = KB < NB ? KB : NB - 1;
        if (dot) {
            int g = 4 * KB + q4;
            g = g < d32 ? g : d32 - 1;
            const uintptr_t base = copy2 + 8 * ((uintptr_t)g * (uintptr_t)n_pad + (uintptr_t)row0 + (uintptr_t)n16);
#pragma unroll
            for (int sl = 0; sl < NSL; ++sl) {
                const pair_t v = __builtin_nontemporal_load(
                    (const __attribute__((address_space(1))) pair_t *)(base + (uintptr_t)(8 * 16 * sl)));
                dst[2 * sl] = v[0];
                dst[2 * sl + 1] = v[1];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int m = 0; m < TM; ++m)
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) {
                    int g = 2 * (2 * KB + j) + (sl >> 1);
                    g = g < d32 ? g : d32 - 1;
                    const uintptr_t rg = (uintptr_t)(row0 >> 5) + (uintptr_t)(2 * m + (q4 >> 1));
                    const uintptr_t unit = ((uintptr_t)g * (uintptr_t)n32 + rg) * 32 + (uintptr_t)(16 * (sl & 1) + n16);
                    dst[(j * TM + m) * 4 + sl] = __builtin_nontemporal_load(
                        (const __attribute__((address_space(1))) uint32_t *)(copy1 + 8 * unit + (uintptr_t)(4 * (q4 & 1))));
                }
        }
    };

    const int64_t t_end = a.step0 + a.nsteps;
    if (p < NT) issue(a.step0 * a.B + TS * (int64_t)p, 0, buf0);
    for (int64_t t = a.step0; t < t_end; ++t) {
        // ============ the model of this step: y_j = delta_j x_j, its largest magnitude, sum_j mid_j x_j
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
        __syncthreads();
        if (lane == 0) { red[wave] = ymax; red[kWaves + wave] = cqp; }
        __syncthreads();
        float cq = 0.0f;
        ymax = 0.0f;
#pragma unroll
        for (int v = 0; v < kWaves; ++v) { ymax = fmaxf(ymax, red[v]); cq += red[kWaves + v]; }
        const int ky = scale_exponent(ymax, 29);
        // digits: a thread writes one dword (8 nibbles) of each of the 16 rows.  Dword D of a block:
        // lane group q = D / 4 (features 32 q ..), operand dword D % 4, whose nibble i is the code
        // 16 (dword / 2) + dword % 2 + 2 i of the packed unit -- the order the expansion below gives.
        for (int o = tid; o < NB * 16; o += kThreads) {
            const int blk = o >> 4, D = o & 15, q = D >> 2, dw = D & 3;
            uint32_t rows[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) rows[k] = 0u;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int f = blk * 128 + 32 * q + 16 * (dw >> 1) + (dw & 1) + 2 * i;
                const int Y = f < nfeat ? __float2int_rn(ldexpf(gs[f], ky)) : 0;
                const uint32_t Yb = (uint32_t)Y + 0x2AAAAAAAu;          // every digit + 2: |Y| < 2^29
#pragma unroll
                for (int k = 0; k < 15; ++k)                           // digits -2, -1, 0, 1 as E2M1: C, A, 0, 2
                    rows[k] |= ((0x20ACu >> (4 * ((Yb >> (2 * k)) & 3u))) & 0xFu) << (4 * i);
                rows[15] |= (((Yb >> 30) & 1u) * 2u) << (4 * i);       // the carry out of digit 14: 0 or 1
            }
#pragma unroll
            for (int k = 0; k < 16; ++k)
                *reinterpret_cast<uint32_t *>(ydig + (size_t)blk * 1024 + (k * 4 + q) * 16 + dw * 4) = rows[k];
        }
        __syncthreads();                       // (the digits are read from gs: clear it afterwards)
        for (int j = tid; j < nfeat; j += kThreads) gs[j] = 0.0f;
        float rtot = 0.0f;
        __syncthreads();

        // ============ tiles of 64 TM samples, dealt out in turn: dot pass, residuals, gradient pass
        for (int64_t T = p; T < NT; T += P) {
            const int64_t row0 = t * a.B + TS * T;
            const int64_t row_next = T + P < NT ? row0 + TS * (int64_t)P
                                     : t + 1 < t_end ? (t + 1) * a.B + TS * (int64_t)p : row0;
            float label[TM];
#pragma unroll
            for (int m = 0; m < TM; ++m) label[m] = a.b[row0 + 64 * m + lane];
            v4f acc[NSL];
#pragma unroll
            for (int sl = 0; sl < NSL; ++sl) acc[sl] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
            // Digit operands of the gradient pass, taken from LDS once per tile: block m of the
            // residuals for tile slot sl is the digits in the lanes of that slot, zeros elsewhere.
            // (Read per matrix instruction, as k_sgd_rows does, the digits are 16 bytes a lane from
            // LDS against 4 bytes of packed codes from memory: at 2 bits that, not the memory, is
            // what the kernel ran at.)  They live when the accumulators of the dot pass no longer do.
            v4i rop[TM][4];
            // one item: request the next one into the other buffer, then compute
            auto item = [&](int s, uint32_t (&cur)[NW], uint32_t (&nxt)[NW]) __attribute__((always_inline)) {
                if (s + 1 < 2 * ND) issue(row0, s + 1, nxt);
                else issue(row_next, 0, nxt);
                if (s == ND) {
                    // ---- residuals of the tile, between the two passes: fold the digit rows
#pragma unroll
                    for (int sl = 0; sl < NSL; ++sl) {
                        // rows 4 q4 .. 4 q4 + 3 of sample 16 sl + n16: exact in fp32 (a few thousand halves)
                        const float S = ((acc[sl][3] * 4.0f + acc[sl][2]) * 4.0f + acc[sl][1]) * 4.0f + acc[sl][0];
                        zq[(wave * TS + 16 * sl + n16) * 4 + q4] = __float2int_rn(2.0f * S);
                    }
                    lds_barrier();
                    if (wave == 0) {
                        float r[TM], rabs = 0.0f;
#pragma unroll
                        for (int m = 0; m < TM; ++m) {
                            long long z = 0;
#pragma unroll
                            for (int v = 0; v < kWaves; ++v) {
                                const v4i part = *reinterpret_cast<const v4i *>(zq + (v * TS + 64 * m + lane) * 4);
                                z += (long long)part[0] + ((long long)part[1] << 8) + ((long long)part[2] << 16) +
                                     ((long long)part[3] << 24);
                            }
                            r[m] = (float)(ldexp((double)z, -ky) + (double)cq) - label[m];
                            rabs = fmaxf(rabs, fabsf(r[m]));
                        }
                        // (the sum of the residuals: blocks of 64 in order, as the tiles of k_sgd_rows)
                        const float rmax = wave_reduce_dpp(rabs, [](float u, float v) { return fmaxf(u, v); });
#pragma unroll
                        for (int m = 0; m < TM; ++m) rtot += wave_sum_dpp(r[m]);
                        const int kr = rmax < 3.0e38f ? scale_exponent(rmax, 29) : 0;
#pragma unroll
                        for (int m = 0; m < TM; ++m)
                            store_digits(rdig + m * 256 + my_pos, signed_digits(__float2int_rn(ldexpf(r[m], kr))));
                        if (lane == 0) misc[0] = kr;
                    }
                    lds_barrier();
#pragma unroll
                    for (int m = 0; m < TM; ++m) {
                        const v4i dg = *reinterpret_cast<const v4i *>(rdig + m * 256 + dig_off);
#pragma unroll
                        for (int sl = 0; sl < 4; ++sl) rop[m][sl] = slot_of == sl ? dg : v4i{0, 0, 0, 0};
                    }
                }
                const int KB = wave + kWaves * (s < ND ? s : s - ND);
                if (s < ND) {
                    if (KB < NB) {
                        const v4i ad = *reinterpret_cast<const v4i *>(ydig + (size_t)KB * 1024 + (n16 * 4 + q4) * 16);
                        const v8i a8 = {ad[0], ad[1], ad[2], ad[3], 0, 0, 0, 0};
#pragma unroll
                        for (int sl = 0; sl < NSL; ++sl) {
                            const uint32_t p0 = cur[2 * sl], p1 = cur[2 * sl + 1];
                            const v8i b8 = {(int)(p0 & 0x33333333u), (int)((p0 >> 2) & 0x33333333u),
                                            (int)(p1 & 0x33333333u), (int)((p1 >> 2) & 0x33333333u), 0, 0, 0, 0};
                            acc[sl] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc[sl], 4, 4, 0, 0, 0, 0);
                        }
                    }
                } else {
                    const int kr = misc[0];
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int kb = 2 * KB + j;
                        if (KB < NB && kb < NKB) {
                            v4i c = {0, 0, 0, 0};
#pragma unroll
                            for (int m = 0; m < TM; ++m)
#pragma unroll
                                for (int sl = 0; sl < 4; ++sl) {
                                    const uint32_t one[1] = {cur[(j * TM + m) * 4 + sl]};
                                    c = __builtin_amdgcn_mfma_i32_16x16x64_i8(rop[m][sl], expand_codes<BITS>(one), c, 0, 0, 0);
                                }
                            gs[kb * 64 + lane] += fixed_to_float(combine_digits(c), kr);
                        }
                    }
                }
            };
            for (int s = 0; s < 2 * ND; s += 2) {
                item(s, buf0, buf1);
                item(s + 1, buf1, buf0);
            }
        }

        // ============ gradients of all workgroups -> model (as k_sgd_rows)
        __syncthreads();
        float *const mine = a.part + (size_t)p * nfeat;
        for (int j = tid; j < nfeat; j += kThreads) store_dev(mine + j, gs[j]);
        if (tid == 0) store_dev(a.part + (size_t)P * nfeat + p, rtot);
        grid_sync();
        {
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
                for (int q0 = q4; q0 < P; q0 += 256) {
                    // (sixteen loads in flight at a time; the additions in the order of k_sgd_rows)
#pragma unroll 1
                    for (int e0 = 0; e0 < 64; e0 += 16) {
                        float v[16];
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int q = q0 + 4 * (e0 + e);
                            v[e] = load_dev(a.part + (size_t)(q < P ? q : P - 1) * nfeat + j);
                        }
#pragma unroll
                        for (int e = 0; e < 16; ++e) s += q0 + 4 * (e0 + e) < P ? v[e] : 0.0f;
                    }
                }
                float rs = (rv[0] + rv[1]) + (rv[2] + rv[3]);
                for (int q = lane + 4 * kWave; q < P; q += kWave) rs += load_dev(rsum_all + q);
                const float Rtot = wave_sum_dpp(rs);
                const float s0 = __shfl(s, n16, kWave), s1 = __shfl(s, 16 + n16, kWave);
                const float s2 = __shfl(s, 32 + n16, kWave), s3 = __shfl(s, 48 + n16, kWave);
                const float G = (s0 + s1) + (s2 + s3);
                if (q4 == 0 && j < a.d) {
                    const float g = __fdiv_rn(a.mid[j] * Rtot + a.dl[j] * G, (float)a.B);
                    const float reg = a.l2 * xj;
                    const float stp = a.lr * (g + reg);
                    const float v = xj - stp;
                    store_dev(a.x + j, a.prox ? apply_prox(v, a.prox, a.lr, a.prox_coef) : v);
                }
            }
        }
        if (t + 1 < t_end) grid_sync();
    }
}

template <int TM>
__global__ __launch_bounds__(kThreads, 1) void k_sgd_rows_fp4(RowsArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    sgd_rows_fp4<TM>(a, smem);
}

}  // namespace zipml
