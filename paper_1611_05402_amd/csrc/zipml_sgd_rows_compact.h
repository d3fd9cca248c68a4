// The sample-owner epoch kernel reading COMPACT records (included by zipml_sgd.hip after
// zipml_sgd_rows.h, whose arguments and host helpers it shares).
//
// Sec. 2.2, "Overhead of Storing Samples": the two quantisations of a value differ by at most one
// level, so a base level and one bit per sample hold both -- b + 2 bits per value instead of 2 b.
// zipml_compact_encode writes that record for the two copies in the sample-major layout (a unit is
// one sample x 32 features: a plane of 8 dwords of base levels a unit, then a plane of one dword
// of bits per copy and unit); here the epoch runs on that record alone, so a step reads
// (b + 2) / 2b of the bytes of the two packed copies: 62.5 % at 8 bits, the only width built.
//
// The dot pass wants copy 2 sample-major: base + bit, as stored.  The gradient pass wants copy 1
// with 16 SAMPLES of one feature in a lane's operand, the transpose of what is stored.  A workgroup
// takes both passes over the same tile of 64 samples, and a wave takes the same 64-feature blocks in
// both, so in the dot pass the wave also writes the bytes of copy 1 of its blocks into a private
// piece of LDS, a sample per 64-byte row, and when the residuals are known it reads them back with
// ds_read_b64_tr_b8, the transposing LDS read of gfx950: 16 lanes name 16 pieces of 8 bytes, and
// the lane 8 p + c of them receives byte c of the pieces 2 j + p, j = 0 .. 7 (found by reading a
// known pattern; test_epoch_on_the_compact_record would fail on any other order).  With a row
// per sample, pieces (sample s + j, features f .. f + 7) in lanes 2 j + p hand lane 8 p + c the
// eight samples of feature f + 8 p + c: half an operand.  The 16-byte quarters of a row are stored
// exclusive-or'ed with bits 1-2 of the row number, which keeps both the 16-byte writes and the
// transposing reads off each other's banks without padding (the areas fill the LDS at d = 2048).
// No packed byte is read twice and the gradient pass reads none at all.
//
// Everything else -- digits of y in LDS, residuals inside the workgroup, exact integer sums on
// v_mfma_i32_16x16x64_i8, the two meetings per step and the fixed-order sum of the per-workgroup
// gradients -- is that of k_sgd_rows, and the sums are the same integers: the model after an epoch
// is bit-identical to the one k_sgd_rows computes from the two packed copies.
#pragma once

namespace zipml {

constexpr int kTurnBytes = 64 * 64;                   // a wave's transpose area for one block: 64 samples x 64 features

// LDS of k_sgd_rows_compact for NKB blocks of 64 features.
__host__ __device__ inline size_t rows_compact_lds_bytes(int NKB)
{
    const int NG = NKB <= 2 * kWaves ? 2 : 4;         // blocks per wave
    return ((rows_lds_bytes(NKB) + 15) & ~(size_t)15) + (size_t)kWaves * NG * kTurnBytes;
}

// 16 bits -> 16 bytes of 0 / 1 (bit 4 k + e of `bits16` to byte e of dword k).
__device__ __forceinline__ v4i spread_bits16(uint32_t bits16)
{
    v4i r;
#pragma unroll
    for (int k = 0; k < 4; ++k)   // 4 bits times (1 + 2^7 + 2^14 + 2^21): bit e lands on bit 8 e
        r[k] = (int)((((bits16 >> (4 * k)) & 0xFu) * 0x00204081u) & 0x01010101u);
    return r;
}

// NG: 64-feature blocks per wave (2 or 4; blocks past the last one are skipped).
template <int NG>
__device__ __forceinline__ void sgd_rows_compact(const RowsArgs &a, unsigned char *smem)
{
    constexpr int HW = 4;                             // dwords of a lane operand: 16 codes of 8 bits
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n16 = lane & 15, q4 = lane >> 4;
    const int P = gridDim.x, p = blockIdx.x;
    const int NKB = a.NKB, nfeat = NKB * 64;
    const int64_t NT = a.B / 64;

    // ---- LDS (as k_sgd_rows, then the transpose areas)
    int8_t *const ydig = (int8_t *)smem;
    float *const gs = (float *)(smem + (size_t)NKB * 256);
    unsigned char *tail = smem + (size_t)NKB * 512;
    long long *const zpart = (long long *)tail;
    int8_t *const rdig = (int8_t *)(tail + kWaves * 64 * 8);
    float *const red = (float *)(tail + kWaves * 64 * 8 + 256);
    int *const misc = (int *)(tail + kWaves * 64 * 8 + 256 + 64);
    int8_t *const zeros = (int8_t *)(tail + kWaves * 64 * 8 + 256 + 128);
    // (addressed as LDS outright: through generic pointers the byte accesses below become flat
    // instructions with an address register pair each, and the kernel spills)
    typedef __attribute__((address_space(3))) unsigned char lds_u8;
    typedef int v2i __attribute__((ext_vector_type(2)));
    typedef __attribute__((address_space(3))) v4i lds_v4;
    typedef __attribute__((address_space(3))) v2i lds_v2;
    lds_u8 *const turn =
        (lds_u8 *)(smem + ((rows_lds_bytes(NKB) + 15) & ~(size_t)15) + (size_t)wave * (NG * kTurnBytes));
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

    const int my_pos = lane;                          // 8-bit codes: digits in natural order
    const int dig_off = (n16 & 3) * 64 + q4 * 16, slot_of = n16 >> 2;
    const int zero_off = (int)(zeros - ydig);
    // transpose areas: quarter q of row r lives at quarter q ^ ((r >> 1) & 3)
    const int wr_quarter = 16 * (q4 ^ ((n16 >> 1) & 3));                   // rows 16 sl + n16
    const int rd_row = (16 * q4 + (n16 >> 1)) * 64 + 8 * (n16 & 1);        // rows 16 q4 [+ 8] + n16 / 2
    const int rd_swz = 16 * ((n16 >> 2) & 3);

    // ---- compact data in flight: two items (one 64-feature block of the tile each) of four lane
    // operands: 4 dwords of base levels, the unit's two dwords of bits
    typedef uint32_t base_t __attribute__((ext_vector_type(4), aligned(16)));
    typedef uint32_t bits_t __attribute__((ext_vector_type(2), aligned(8)));
    uint32_t bufb[2][4][HW], bufu[2][4][2];
    // lane = sample 16 sl + n16 of the tile, half q4 & 1 of feature group 2 kb + q4 / 2.  The base
    // plane is a packed 8-bit array (unit (group, sample) 32 bytes at 32 (group n_pad + sample)); the
    // pairs of bit dwords follow it in the same order, 8 bytes a unit.  A load instruction of the
    // wave covers whole memory lines that no other instruction touches (16 units x 32 bytes of two
    // groups; 16 pairs x 8 bytes = one line of two groups), so the stream can be non-temporal.
    const uintptr_t rec = (uintptr_t)a.p2;            // the compact record
    const uintptr_t pairs = rec + (uintptr_t)32 * (uintptr_t)a.n_pad * (uintptr_t)a.d32;
    const uint32_t lane_base = (uint32_t)(n16 * 32 + (q4 & 1) * 16), lane_pair = (uint32_t)(n16 * 8);
    const int d32 = a.d32;
    auto issue = [&](int64_t row0, int k, int slot) __attribute__((always_inline)) {
        int kb = wave + kWaves * k;
        kb = kb < NKB ? kb : NKB - 1;
        // (a block whose second group is padding reads its first group twice; the digits of y
        // there are zero and its gradient is never used)
        const int g = 2 * kb + ((q4 >> 1) && 2 * kb + 1 < d32 ? 1 : 0);
        const uintptr_t unit = (uintptr_t)g * (uintptr_t)a.n_pad + (uintptr_t)row0;
        const uintptr_t base0 = rec + 32 * unit + lane_base, pair0 = pairs + 8 * unit + lane_pair;
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {
            const base_t vb = __builtin_nontemporal_load(
                (const __attribute__((address_space(1))) base_t *)(base0 + (uintptr_t)(16 * 32 * sl)));
            const bits_t vu = __builtin_nontemporal_load(
                (const __attribute__((address_space(1))) bits_t *)(pair0 + (uintptr_t)(16 * 8 * sl)));
#pragma unroll
            for (int h = 0; h < HW; ++h) bufb[slot][sl][h] = vb[h];
            bufu[slot][sl][0] = vu[0];
            bufu[slot][sl][1] = vu[1];
        }
    };

    const int64_t t_end = a.step0 + a.nsteps;
    if (p < NT) {
        issue(a.step0 * a.B + 64 * (int64_t)p, 0, 0);
        issue(a.step0 * a.B + 64 * (int64_t)p, 1, 1);
    }
    for (int64_t t = a.step0; t < t_end; ++t) {
        // ============ the model of this step: digits of y_j = delta_j x_j, sum_j mid_j x_j
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
        for (int j = tid; j < nfeat; j += kThreads) {
            const int Y = __float2int_rn(ldexpf(gs[j], ky));
            store_digits(ydig + (j >> 6) * 256 + (j & 63), signed_digits(Y));
            gs[j] = 0.0f;
        }
        float rtot = 0.0f;
        __syncthreads();

        // ============ tiles of 64 samples, dealt out in turn.  The gradient pass of a tile runs
        // block by block between the items of the NEXT tile's dot pass (block k of the old tile
        // leaves its transpose area just before item k of the new tile fills it): every item then
        // consumes one buffer and requests one, two items ahead, at an even pace.  With the passes
        // one after the other nothing is requested during a gradient pass and the dot pass waits
        // for its last items from scratch (measured: no faster than reading both packed copies).
        const int rdig_off = (int)(rdig - ydig);
        // item k of a tile's dot pass: copy 2 to the matrix cores, copy 1 into the transpose area
        auto dot_item = [&](int k, int64_t row0, int64_t row_next, v4i &cdot) __attribute__((always_inline)) {
            const int slot = k & 1;
            const int kb = wave + kWaves * k;
            v4i c2b[4];
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                const uint32_t sh = (uint32_t)(q4 & 1) * 16u;
                const v4i u1 = spread_bits16((bufu[slot][sl][0] >> sh) & 0xFFFFu);
                const v4i u2 = spread_bits16((bufu[slot][sl][1] >> sh) & 0xFFFFu);
                v4i c1b;
#pragma unroll
                for (int h = 0; h < HW; ++h) {
                    // (a byte of base plus its bit never carries: the code is at most 255)
                    c2b[sl][h] = (int)((bufb[slot][sl][h] + (uint32_t)u2[h]) ^ 0x80808080u);
                    c1b[h] = (int)((bufb[slot][sl][h] + (uint32_t)u1[h]) ^ 0x80808080u);
                }
                // copy 1: row = sample 16 sl + n16, quarter q4 (features 16 q4 .. + 15) of the block
                *(lds_v4 *)(turn + k * kTurnBytes + (16 * sl + n16) * 64 + wr_quarter) = c1b;
            }
            // the buffer is free: request the item two ahead
            if (k + 2 < NG) issue(row0, k + 2, slot);
            else issue(row_next, k + 2 - NG, slot);
            if (kb < NKB) {
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) {
                    const v4i ad = *reinterpret_cast<const v4i *>(
                        ydig + (slot_of == sl ? kb * 256 + dig_off : zero_off));
                    cdot = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad, c2b[sl], cdot, 0, 0, 0);
                }
            }
        };
        // block k of the gradient pass of the tile whose residual digits are in LDS
        auto grad_block = [&](int k, int kr) __attribute__((always_inline)) {
            const int kb = wave + kWaves * k;
            if (kb < NKB) {
                v4i c = {0, 0, 0, 0};
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) {
                    // operand: feature 16 sl + n16 of samples 16 q4 .. 16 q4 + 15.  This lane names
                    // the piece (sample 16 q4 + n16 / 2 [+ 8], features 16 sl + 8 (n16 & 1) ..).
                    const lds_u8 *piece = turn + k * kTurnBytes + rd_row + ((16 * sl) ^ rd_swz);
                    const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2 *)piece);
                    const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2 *)(piece + 8 * 64));
                    const v4i op = {lo[0], lo[1], hi[0], hi[1]};
                    const v4i ad = *reinterpret_cast<const v4i *>(
                        ydig + (slot_of == sl ? rdig_off + dig_off : zero_off));
                    c = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad, op, c, 0, 0, 0);
                }
                gs[kb * 64 + lane] += fixed_to_float(combine_digits(c), kr);
            }
        };
        bool pending = false;                  // a tile's gradient pass is still to run
        int kr_pending = 0;
        for (int64_t T = p; T < NT; T += P) {
            const int64_t row0 = t * a.B + 64 * T;
            // (after the last tile of a step: the first tile of the next step; after the last step:
            // this tile again, never used)
            const int64_t row_next = T + P < NT ? row0 + 64 * (int64_t)P
                                     : t + 1 < t_end ? (t + 1) * a.B + 64 * (int64_t)p : row0;
            const float label = a.b[row0 + lane];
            v4i cdot = {0, 0, 0, 0};
            if (pending) {
#pragma unroll
                for (int k = 0; k < NG; ++k) {
                    // (a wave's LDS instructions execute in the order they are issued: the reads of
                    // area k are done when item k writes it)
                    grad_block(k, kr_pending);
                    dot_item(k, row0, row_next, cdot);
                }
            } else {
#pragma unroll
                for (int k = 0; k < NG; ++k) dot_item(k, row0, row_next, cdot);
            }
            // ---- residuals of the tile (wave 0); every wave is past the old tile's gradient pass
            zpart[wave * 64 + lane] = combine_digits(cdot);
            lds_barrier();
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
            kr_pending = misc[0];
            pending = true;
        }
        if (pending) {
#pragma unroll
            for (int k = 0; k < NG; ++k) grad_block(k, kr_pending);
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
                    // (sixteen loads in flight at a time; the additions run in the same order as in
                    // k_sgd_rows, which has all 64 in flight)
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

template <int NG>
__global__ __launch_bounds__(kThreads, 1) void k_sgd_rows_compact(RowsArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    sgd_rows_compact<NG>(a, smem);
}

}  // namespace zipml
