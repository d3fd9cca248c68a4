// zipml_sgd_epoch / zipml_debug_step: double-sampled minibatch SGD on packed low-bit data.
//
// Method: Sec. 2.2 eq. (5), g = mean_i Q1(a_i)(Q2(a_i)^T x - b_i); end-to-end variant of Supp. C-E.
//
// Decomposition (feature-owner): workgroup w owns a block of 32*GQ features for the whole epoch and
// keeps its slice of the model in LDS.  Per step it
//   1. streams its slice of copy 2 (sample-major units) and adds the partial dot products of the
//      `batch` samples into a device-wide accumulator,
//   2. meets the other workgroups at ONE grid-wide barrier,
//   3. reads the `batch` residuals, streams its slice of copy 1 (feature-major units), forms its
//      slice of the mean gradient and updates its slice of the model -- all locally.
// The packed data does not depend on the model, so the slice for step t+1 is fetched straight into
// LDS (global_load_lds) while step t waits at the barrier.
// End-to-end mode adds two small exchanges per step (the l2 norms of model and gradient).
#include "zipml_device.h"
#include "zipml_host.h"

#include <math.h>

namespace zipml {

constexpr int kThreads = 256;
constexpr uint32_t kSpinLimit = 1u << 22;   // bounded wait: a lost workgroup ends in ZIPML_ETIMEOUT

struct SgdArgs {
    const uint32_t *p1, *p2;
    const float *levels;
    const uint16_t *grid;
    const float *b;
    float *x;
    int64_t n_pad, n32;
    int d, d32;
    int B;                 // batch
    int64_t step0;         // first step of this launch
    int nsteps;
    float lr, grid_lo, grid_step;
    int grad_bits, model_bits;
    int ident_grid;        // grid_idx[j][c] == c
    uint64_t seed;
    uint32_t epoch;
    int GQ, W;             // feature groups per workgroup, workgroups
    int seg_first, seg_last;   // segments of a step run by this launch (0..3)
    int persistent;        // 1: segments are separated by in-kernel grid barriers
    int depth;             // LDS slots for packed data
    int slot_bytes;
    // workspace
    int *status;
    uint32_t *sync;
    double *nrm;           // [2 kinds][2 slots][512]
    float *acc;            // [3][acc_words]
    int acc_words;
    float *gbuf;           // [d_pad] gradient carried between launches (stepwise, grad_bits > 0)
    // debug outputs (may be null)
    int32_t *dbg_m, *dbg_acc, *dbg_gq;
    float *dbg_r, *dbg_g;
};

// ---------------------------------------------------------------------------------------------
// Grid-wide barrier: one monotonically increasing arrival counter.  Data exchanged across it is
// written and read with device-scope accesses only (add_dev / store_dev / load_dev).
// ---------------------------------------------------------------------------------------------
struct GridBarrier {
    uint32_t *ctr;
    int *status;
    uint32_t W;
    uint32_t passed;   // barriers completed so far
    bool dead;

    __device__ void arrive_and_wait()
    {
        release_dev();           // this wave's device-scope writes are performed
        __syncthreads();
        ++passed;
        if (threadIdx.x == 0) {
            add_dev(ctr, 1u);
            const uint32_t target = passed * W;
            uint32_t spins = 0;
            while (!dead && load_dev(ctr) < target) {
                __builtin_amdgcn_s_sleep(1);
                if (++spins > kSpinLimit) {
                    store_dev(status, (int)ZIPML_ETIMEOUT);
                    dead = true;
                }
            }
        }
        __syncthreads();
    }
};

// Adjacent-pair tree sum of `len` (power of two) doubles in LDS; result in a[0].
__device__ __forceinline__ void lds_tree_sum(double *a, int len)
{
    for (int stride = 1; stride < len; stride <<= 1) {
        __syncthreads();
        for (int i = threadIdx.x * 2 * stride; i + stride < len; i += kThreads * 2 * stride)
            a[i] = a[i] + a[i + stride];
    }
    __syncthreads();
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

// Asynchronous copy of `dwords` (multiple of 4) dwords from global to LDS, 16 B per lane,
// issued by the whole workgroup.  Completion: s_waitcnt vmcnt(0) in every wave, then a barrier.
__device__ __forceinline__ void async_copy(const uint32_t *__restrict__ src, uint32_t *dst_lds,
                                           int dwords)
{
    const int chunks = dwords >> 2;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave_first = threadIdx.x - lane;
    for (int c0 = 0; c0 < chunks; c0 += kThreads) {
        const int c = c0 + wave_first + lane;
        if (c0 + wave_first < chunks) {
            uint32_t *wave_dst = dst_lds + (size_t)(c0 + wave_first) * 4;
            if (c < chunks)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void *)(src + (size_t)c * 4),
                    (__attribute__((address_space(3))) void *)wave_dst, 16, 0, 0);
        }
    }
}

__device__ __forceinline__ void async_wait_all()
{
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
}

template <int BITS>
__device__ __forceinline__ void lds_unit(const uint32_t *p, uint32_t (&u)[BITS])
{
#pragma unroll
    for (int q = 0; q < BITS; ++q) u[q] = p[q];
}

// ---------------------------------------------------------------------------------------------
// The epoch kernel.
// ---------------------------------------------------------------------------------------------
template <int BITS>
__global__ __launch_bounds__(kThreads) void k_sgd(SgdArgs a)
{
    constexpr int K = 1 << BITS;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int w = blockIdx.x;
    const int CW = 32 * a.GQ;
    const int B = a.B;
    const int nrg = B >= 32 ? B / 32 : 1;          // sample groups per step
    const int Rlen = nrg * 32;                     // residual slots (zero outside the batch)
    const bool int_mode = a.model_bits > 0;
    const bool seq_grad = int_mode;                // gradient in a fixed fp32 order
    const int j0 = w * CW;                         // first feature of this workgroup

    // ---- LDS carve
    size_t off = 0;
    auto carve = [&](size_t bytes) { void *p = smem + off; off += (bytes + 15) & ~(size_t)15; return p; };
    // the packed-data slots come first so that their LDS addresses stay below 64 KiB
    uint32_t *ring = (uint32_t *)carve((size_t)a.depth * a.slot_bytes);
    float *Ls = (float *)carve((size_t)CW * K * 4);
    uint16_t *Gs = (uint16_t *)carve(int_mode && !a.ident_grid ? (size_t)CW * K * 2 : 0);
    float *xs = (float *)carve(CW * 4);
    float *ys = (float *)carve(CW * 4);
    float *los = (float *)carve(CW * 4);
    float *dls = (float *)carve(CW * 4);
    float *gs = (float *)carve(CW * 4);
    int *ms = (int *)carve(CW * 4);
    float *rs = (float *)carve((size_t)Rlen * 4);
    float *gpart = (float *)carve(kThreads * 4);
    double *red = (double *)carve(512 * 8);
    float *fscr = (float *)carve(16 * 4);

    // ---- one-time set-up: level slice, model slice
    for (int e = tid; e < CW * K; e += kThreads) {
        const int jj = e / K, j = j0 + jj;
        Ls[e] = j < a.d ? a.levels[(size_t)j * K + (e % K)] : 0.0f;
        if (int_mode && !a.ident_grid) Gs[e] = j < a.d ? a.grid[(size_t)j * K + (e % K)] : (uint16_t)0;
    }
    for (int c = tid; c < CW; c += kThreads) xs[c] = (j0 + c < a.d) ? a.x[j0 + c] : 0.0f;
    __syncthreads();
    // Are the levels of every owned feature evenly spaced (fp64 formula, rounded once)?  Then a
    // value is lo + code * delta and the table look-up is replaced by arithmetic.
    int ok = 1;
    for (int e = tid; e < CW * K; e += kThreads) {
        const int jj = e / K, c = e % K;
        const double lo = (double)Ls[jj * K], wdt = (double)Ls[jj * K + K - 1] - lo;
        ok &= (Ls[e] == (float)(lo + ((double)c * wdt) / (double)(K - 1)));
    }
    const bool affine = __syncthreads_and(ok) && !int_mode;
    for (int c = tid; c < CW; c += kThreads) {
        los[c] = Ls[c * K];
        dls[c] = (float)(((double)Ls[c * K + K - 1] - (double)Ls[c * K]) / (double)(K - 1));
        ys[c] = dls[c] * xs[c];
        gs[c] = 0.0f;
        ms[c] = 0;
    }
    for (int i = tid; i < Rlen; i += kThreads) rs[i] = 0.0f;
    __syncthreads();
    float Cq = 0.0f;   // sum_j lo_j x_j over the owned features (affine mode)
    if (affine) Cq = block_sum<float>(tid < CW ? los[tid] * xs[tid] : 0.0f, fscr);

    GridBarrier bar{a.sync, a.status, (uint32_t)a.W, 0u, false};

    // ---- packed-data slots
    const int r2_dw = B * BITS;                 // one feature group of copy 2 for one step
    const int r1_dw = nrg * 32 * BITS;          // one feature group of copy 1 for one step
    const int b_dw = (B + 3) & ~3;
    const int slot_dw = a.slot_bytes / 4;
    auto fetch = [&](int64_t t, int slot) {
        uint32_t *s = ring + (size_t)slot * slot_dw;
        for (int gq = 0; gq < a.GQ; ++gq) {
            const int64_t g = (int64_t)w * a.GQ + gq;
            if (g >= a.d32) break;
            async_copy(a.p2 + (g * a.n_pad + t * B) * BITS, s + gq * r2_dw, r2_dw);
            async_copy(a.p1 + ((g * a.n32 + (t * B) / 32) * 32) * BITS,
                       s + a.GQ * r2_dw + gq * r1_dw, r1_dw);
        }
        async_copy((const uint32_t *)(a.b + t * B), s + a.GQ * (r2_dw + r1_dw), b_dw);
    };
    const int64_t t_end = a.step0 + a.nsteps;
    fetch(a.step0, 0);

    for (int64_t t = a.step0; t < t_end; ++t) {
        const int it = (int)(t - a.step0);
        const int slot = it % a.depth;
        const uint32_t *S = ring + (size_t)slot * slot_dw;
        const uint32_t *S2 = S, *S1 = S + a.GQ * r2_dw;
        const float *bS = (const float *)(S + a.GQ * (r2_dw + r1_dw));
        float *accf = a.acc + (size_t)(t % 3) * a.acc_words;
        int *acci = (int *)accf;

        async_wait_all();                                    // slot `slot` has landed
        if (a.persistent && t + 1 < t_end) fetch(t + 1, (it + 1) % a.depth);

        // ================= segment 0: ||x||_2 partial (model quantisation only) =================
        float Mx = 0.0f, sigma = 0.0f;
        const int s_m = (1 << (a.model_bits > 0 ? a.model_bits - 1 : 1)) - 1;
        double *nx = a.nrm + (size_t)(t & 1) * 512;
        if (int_mode && a.seg_first <= 0) {
            if (tid < CW) red[tid] = (double)xs[tid] * (double)xs[tid];
            lds_tree_sum(red, CW);
            if (tid == 0) store_dev(nx + w, red[0]);
            if (a.persistent) bar.arrive_and_wait();
        }
        if (a.seg_last < 1) continue;

        // ================= segment 1: model codes, dot pass =====================================
        if (a.seg_first <= 1) {
            if (int_mode) {
                int Wp = 1;
                while (Wp < a.W) Wp <<= 1;
                for (int i = tid; i < Wp; i += kThreads) red[i] = i < a.W ? load_dev(nx + i) : 0.0;
                lds_tree_sum(red, Wp);
                Mx = (float)sqrt(red[0]);
                sigma = Mx > 0.0f ? __fdiv_rn(Mx, (float)s_m) : 0.0f;
                __syncthreads();
                int mine = 0;
                if (tid < CW) {
                    const int j = j0 + tid;
                    if (j < a.d) {
                        const Philox4 r = philox_block(a.seed, a.epoch, (uint64_t)t, (uint32_t)j >> 2, 3u);
                        mine = qvec_code(xs[tid], Mx, s_m, u24(r.w[j & 3]));
                    }
                    ms[tid] = mine;
                    if (a.dbg_m && j < a.d) a.dbg_m[j] = mine;
                }
                const int part = block_sum<int>(mine, (int *)fscr);   // also publishes ms[]
                if (tid == 0 && part != 0) add_dev(acci + B, part);
            }
            // dot pass: one sample per thread, all owned feature groups
            for (int i = tid; i < B; i += kThreads) {
                float pf = Cq;
                int pi = 0;
                for (int gq = 0; gq < a.GQ; ++gq) {
                    if ((int64_t)w * a.GQ + gq >= a.d32) break;
                    uint32_t u[BITS];
                    lds_unit<BITS>(S2 + (size_t)(gq * B + i) * BITS, u);
                    const int jb = gq * 32;
#pragma unroll
                    for (int k = 0; k < 32; ++k) {
                        const uint32_t code = unit_code<BITS>(u, k);
                        if (int_mode) {
                            const int gidx = a.ident_grid ? (int)code : (int)Gs[(jb + k) * K + code];
                            pi += gidx * ms[jb + k];
                        } else if (affine) {
                            pf = fmaf((float)code, ys[jb + k], pf);
                        } else {
                            pf = fmaf(Ls[(jb + k) * K + code], xs[jb + k], pf);
                        }
                    }
                }
                if (int_mode) add_dev(acci + i, pi);
                else add_dev(accf + i, pf);
            }
            if (a.persistent) bar.arrive_and_wait();
        }
        if (a.seg_last < 2) continue;

        // ================= segment 2: residuals, gradient pass ==================================
        if (a.seg_first <= 2) {
            if (int_mode && a.seg_first == 2) {
                // stepwise launch: recompute the scale of the model quantiser
                int Wp = 1;
                while (Wp < a.W) Wp <<= 1;
                for (int i = tid; i < Wp; i += kThreads) red[i] = i < a.W ? load_dev(nx + i) : 0.0;
                lds_tree_sum(red, Wp);
                Mx = (float)sqrt(red[0]);
                sigma = Mx > 0.0f ? __fdiv_rn(Mx, (float)s_m) : 0.0f;
                __syncthreads();
            }
            // the accumulator of step t+2 is free once every workgroup has passed this point of
            // step t-1; workgroup 0 clears it now
            if (a.persistent && w == 0) {
                float *nxt = a.acc + (size_t)((t + 2) % 3) * a.acc_words;
                for (int i = tid; i < B + 1; i += kThreads) store_dev(nxt + i, 0.0f);
            }
            const int k0 = B >= 32 ? 0 : (int)((t * B) % 32);   // batch offset inside the sample group
            double summ = 0.0;
            if (int_mode) summ = (double)load_dev(acci + B);
            float rsum = 0.0f;
            for (int i = tid; i < B; i += kThreads) {
                float r;
                if (int_mode) {
                    const int av = load_dev(acci + i);
                    const double z = (double)sigma * ((double)a.grid_lo * summ +
                                                      (double)a.grid_step * (double)av);
                    r = (float)z - bS[i];
                    if (a.dbg_acc && w == 0) a.dbg_acc[i] = av;
                } else {
                    r = load_dev(accf + i) - bS[i];
                }
                rs[k0 + i] = r;
                rsum += r;
                if (a.dbg_r && w == 0) a.dbg_r[i] = r;
            }
            float Rtot = 0.0f;
            if (affine) Rtot = block_sum<float>(rsum, fscr);
            __syncthreads();

            if (seq_grad) {
                // fixed order: one feature per thread, samples in batch order, fp32 fma chain
                if (tid < CW) {
                    const int gq = tid >> 5, cin = tid & 31;
                    float acc = 0.0f;
                    if ((int64_t)w * a.GQ + gq < a.d32) {
                        for (int rgl = 0; rgl < nrg; ++rgl) {
                            uint32_t u[BITS];
                            lds_unit<BITS>(S1 + (size_t)gq * r1_dw + (size_t)(rgl * 32 + cin) * BITS, u);
#pragma unroll
                            for (int k = 0; k < 32; ++k) {
                                if (B < 32 && (k < k0 || k >= k0 + B)) continue;
                                acc = fmaf(Ls[tid * K + unit_code<BITS>(u, k)], rs[rgl * 32 + k], acc);
                            }
                        }
                    }
                    const float g = (j0 + tid < a.d) ? __fdiv_rn(acc, (float)B) : 0.0f;
                    gs[tid] = g;
                    if (a.dbg_g && j0 + tid < a.d) a.dbg_g[j0 + tid] = g;
                }
            } else {
                // free order: (feature, slice of the sample groups) per thread, then reduce slices
                const int nsl = kThreads / CW;
                const int c = tid % CW, sl = tid / CW;
                const int gq = c >> 5, cin = c & 31;
                float acc = 0.0f;
                if (sl < nsl && (int64_t)w * a.GQ + gq < a.d32) {
                    for (int rgl = sl; rgl < nrg; rgl += nsl) {
                        uint32_t u[BITS];
                        lds_unit<BITS>(S1 + (size_t)gq * r1_dw + (size_t)(rgl * 32 + cin) * BITS, u);
                        const float *rr = rs + rgl * 32;
#pragma unroll
                        for (int k = 0; k < 32; ++k) {
                            const uint32_t code = unit_code<BITS>(u, k);
                            if (affine) acc = fmaf((float)code, rr[k], acc);
                            else acc = fmaf(Ls[c * K + code], rr[k], acc);
                        }
                    }
                }
                gpart[tid] = acc;
                __syncthreads();
                if (tid < CW) {
                    float sacc = 0.0f;
                    for (int q = 0; q < nsl; ++q) sacc += gpart[q * CW + tid];
                    float g = affine ? (los[tid] * Rtot + dls[tid] * sacc) : sacc;
                    g = (j0 + tid < a.d) ? g / (float)B : 0.0f;
                    gs[tid] = g;
                    if (a.dbg_g && j0 + tid < a.d) a.dbg_g[j0 + tid] = g;
                }
            }
            __syncthreads();
            // clear the residual slots that belong to this (short) batch for the next step
            if (B < 32) for (int i = tid; i < B; i += kThreads) rs[k0 + i] = 0.0f;
            if (a.grad_bits > 0) {
                double *ng = a.nrm + 1024 + (size_t)(t & 1) * 512;
                if (tid < CW) red[tid] = (double)gs[tid] * (double)gs[tid];
                lds_tree_sum(red, CW);
                if (tid == 0) store_dev(ng + w, red[0]);
                if (!a.persistent && tid < CW && j0 + tid < a.d) a.gbuf[j0 + tid] = gs[tid];
                if (a.persistent) bar.arrive_and_wait();
            }
        }
        if (a.seg_last < 3) continue;

        // ================= segment 3: gradient quantisation, update ==============================
        {
            if (a.grad_bits > 0) {
                if (!a.persistent && a.seg_first == 3 && tid < CW)
                    gs[tid] = (j0 + tid < a.d) ? a.gbuf[j0 + tid] : 0.0f;
                double *ng = a.nrm + 1024 + (size_t)(t & 1) * 512;
                int Wp = 1;
                while (Wp < a.W) Wp <<= 1;
                __syncthreads();
                for (int i = tid; i < Wp; i += kThreads) red[i] = i < a.W ? load_dev(ng + i) : 0.0;
                lds_tree_sum(red, Wp);
                const float Mg = (float)sqrt(red[0]);
                const int s_g = (1 << (a.grad_bits - 1)) - 1;
                const float sg = Mg > 0.0f ? __fdiv_rn(Mg, (float)s_g) : 0.0f;
                if (tid < CW) {
                    const int j = j0 + tid;
                    if (j < a.d) {
                        const Philox4 r = philox_block(a.seed, a.epoch, (uint64_t)t, (uint32_t)j >> 2, 4u);
                        const int code = qvec_code(gs[tid], Mg, s_g, u24(r.w[j & 3]));
                        if (a.dbg_gq) a.dbg_gq[j] = code;
                        const float gh = sg * (float)code;
                        const float stp = a.lr * gh;
                        xs[tid] = xs[tid] - stp;
                    }
                }
            } else if (tid < CW) {
                const float stp = a.lr * gs[tid];
                xs[tid] = xs[tid] - stp;
            }
            __syncthreads();
            if (affine) {
                if (tid < CW) ys[tid] = dls[tid] * xs[tid];
                Cq = block_sum<float>(tid < CW ? los[tid] * xs[tid] : 0.0f, fscr);
            }
            __syncthreads();
        }
    }
    // ---- write the model slice back
    if (a.seg_last >= 3)
        for (int c = tid; c < CW; c += kThreads)
            if (j0 + c < a.d) a.x[j0 + c] = xs[c];
}

// Clears the barrier counter, the status word and the three accumulators.
__global__ void k_sgd_reset(int *status, uint32_t *sync, float *acc, int words, int clear_status)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) { sync[0] = 0u; if (clear_status) status[0] = 0; }
    if (i < words) acc[i] = 0.0f;
}

struct Plan {
    int GQ, W, depth, slot_bytes;
    size_t shmem;
};

static int device_limits(int &cus, int &lds)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ZIPML_ELAUNCH;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess)
        return ZIPML_ELAUNCH;
    return ZIPML_OK;
}

static int make_plan(int64_t d32, int bits, int64_t batch, bool int_table, Plan &p)
{
    int cus = 0, lds = 0;
    if (int rc = device_limits(cus, lds)) return rc;
    const int K = 1 << bits;
    int GQ = 1;
    while ((d32 + GQ - 1) / GQ > cus && GQ < 8) GQ <<= 1;
    if ((d32 + GQ - 1) / GQ > cus) return ZIPML_EUNSUPPORTED;       // d > 32 * 8 * CUs
    p.GQ = GQ;
    p.W = (int)((d32 + GQ - 1) / GQ);
    if (p.W > 512) return ZIPML_EUNSUPPORTED;
    const int CW = 32 * GQ;
    const int nrg = batch >= 32 ? (int)(batch / 32) : 1;
    auto up = [](size_t v) { return (v + 15) & ~(size_t)15; };
    size_t fixed = up((size_t)CW * K * 4) + (int_table ? up((size_t)CW * K * 2) : 0) +
                   6 * up((size_t)CW * 4) + up((size_t)nrg * 32 * 4) + up(kThreads * 4) +
                   up(512 * 8) + up(16 * 4);
    const size_t slot = (size_t)GQ * ((size_t)batch * bits + (size_t)nrg * 32 * bits) * 4 +
                        (size_t)((batch + 3) & ~3) * 4;
    p.slot_bytes = (int)up(slot);
    // two slots (this step and the next); the slots must stay within the first 64 KiB of LDS
    if (fixed + 2 * (size_t)p.slot_bytes > (size_t)lds || 2 * (size_t)p.slot_bytes > 65536)
        return ZIPML_EUNSUPPORTED;   // batch too large for the persistent kernel
    p.depth = 2;
    p.shmem = fixed + (size_t)p.depth * p.slot_bytes;
    return ZIPML_OK;
}

template <int BITS>
static int launch_sgd(hipStream_t s, SgdArgs &a, const Plan &p, bool stepwise)
{
    auto kern = k_sgd<BITS>;
    if (HIP_FAILED(hipFuncSetAttribute((const void *)kern,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.shmem)))
        return ZIPML_ELAUNCH;
    const int words = 3 * a.acc_words;
    hipLaunchKernelGGL(k_sgd_reset, dim3((words + 255) / 256), dim3(256), 0, s, a.status, a.sync,
                       a.acc, words, 1);
    if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    if (!stepwise) {
        a.persistent = 1;
        a.seg_first = 0;
        a.seg_last = 3;
        void *params[] = {&a};
        if (HIP_FAILED(hipLaunchCooperativeKernel((const void *)kern, dim3(a.W), dim3(kThreads),
                                                  params, (unsigned)p.shmem, s)))
            return ZIPML_ELAUNCH;
        return ZIPML_OK;
    }
    // stepwise: every segment of every step is its own launch; kernel boundaries replace barriers
    const int64_t first = a.step0, count = a.nsteps;
    a.persistent = 0;
    a.nsteps = 1;
    for (int64_t t = first; t < first + count; ++t) {
        a.step0 = t;
        // the accumulator that step t uses was last used by step t-3: clear it
        float *accf = a.acc + (size_t)(t % 3) * a.acc_words;
        hipLaunchKernelGGL(k_sgd_reset, dim3((a.acc_words + 255) / 256), dim3(256), 0, s, a.status,
                           a.sync, accf, a.acc_words, 0);
        for (int seg = 0; seg <= 3; ++seg) {
            if (seg == 0 && a.model_bits == 0) continue;
            if (seg == 3 && a.grad_bits == 0) continue;
            a.seg_first = seg;
            a.seg_last = seg;
            if (seg == 2 && a.grad_bits == 0) a.seg_last = 3;
            hipLaunchKernelGGL(kern, dim3(a.W), dim3(kThreads), p.shmem, s, a);
            if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
        }
    }
    return ZIPML_OK;
}

static int run_sgd(void *stream, const void *packed1_dev, const void *packed2_dev,
                   const float *levels_dev, const uint16_t *grid_idx_dev, float grid_lo,
                   float grid_step, int grid_max, const float *b_dev, int64_t n, int64_t d, int bits,
                   float *x_dev, int64_t batch, float lr, int grad_bits, int model_bits,
                   uint64_t seed, uint32_t epoch, int flags, int64_t step0, int64_t nsteps,
                   int32_t *dbg_m, int32_t *dbg_acc, float *dbg_r, float *dbg_g, int32_t *dbg_gq,
                   void *workspace_dev, size_t workspace_bytes)
{
    if (!packed1_dev || !packed2_dev || !levels_dev || !b_dev || !x_dev) return ZIPML_EINVAL;
    if (n <= 0 || d <= 0 || !valid_bits(bits) || batch <= 0 || n % batch != 0) return ZIPML_EINVAL;
    if (!(batch == 4 || batch == 8 || batch == 16 || batch % 32 == 0)) return ZIPML_EINVAL;
    if (n > (int64_t)1 << 40 || d > (1 << 24)) return ZIPML_EINVAL;
    if (model_bits != 0 && (model_bits < 2 || model_bits > 8)) return ZIPML_EINVAL;
    if (grad_bits != 0 && (grad_bits < 2 || grad_bits > 8)) return ZIPML_EINVAL;
    if (epoch >= (1u << 24)) return ZIPML_EINVAL;
    if (step0 < 0 || nsteps < 0 || step0 + nsteps > n / batch) return ZIPML_EINVAL;
    if (flags & ~(ZIPML_SGD_STEPWISE | ZIPML_SGD_AVERAGED)) return ZIPML_EINVAL;
    if (flags & ZIPML_SGD_AVERAGED) return ZIPML_EUNSUPPORTED;
    if (grad_bits > 0 && model_bits == 0) return ZIPML_EUNSUPPORTED;
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

    const Layout lay = make_layout(n, d, bits);
    const bool ident = model_bits > 0 && grid_max == (1 << bits) - 1;
    Plan p;
    if (int rc = make_plan(lay.d32, bits, batch, model_bits > 0 && !ident, p)) return rc;

    unsigned char *ws = (unsigned char *)workspace_dev;
    SgdArgs a{};
    a.p1 = (const uint32_t *)packed1_dev;
    a.p2 = (const uint32_t *)packed2_dev;
    a.levels = levels_dev;
    a.grid = grid_idx_dev;
    a.b = b_dev;
    a.x = x_dev;
    a.n_pad = lay.n_pad;
    a.n32 = lay.n32;
    a.d = (int)d;
    a.d32 = (int)lay.d32;
    a.B = (int)batch;
    a.step0 = step0;
    a.nsteps = (int)nsteps;
    a.lr = lr;
    a.grid_lo = grid_lo;
    a.grid_step = grid_step;
    a.grad_bits = grad_bits;
    a.model_bits = model_bits;
    a.ident_grid = ident ? 1 : 0;
    a.seed = seed;
    a.epoch = epoch;
    a.GQ = p.GQ;
    a.W = p.W;
    a.depth = p.depth;
    a.slot_bytes = p.slot_bytes;
    a.status = (int *)(ws + Workspace::kStatus);
    a.sync = (uint32_t *)(ws + Workspace::kSync);
    a.nrm = (double *)(ws + Workspace::kNorm);
    a.acc = (float *)(ws + Workspace::kAcc);
    a.acc_words = (int)Workspace::acc_words(batch);
    a.gbuf = (float *)(ws + Workspace::sgd_bytes(batch));
    a.dbg_m = dbg_m; a.dbg_acc = dbg_acc; a.dbg_r = dbg_r; a.dbg_g = dbg_g; a.dbg_gq = dbg_gq;
    hipStream_t s = entry_stream(stream);
    const bool stepwise = (flags & ZIPML_SGD_STEPWISE) != 0;
    switch (bits) {
        case 1: return launch_sgd<1>(s, a, p, stepwise);
        case 2: return launch_sgd<2>(s, a, p, stepwise);
        case 3: return launch_sgd<3>(s, a, p, stepwise);
        case 4: return launch_sgd<4>(s, a, p, stepwise);
        case 5: return launch_sgd<5>(s, a, p, stepwise);
        case 6: return launch_sgd<6>(s, a, p, stepwise);
        case 7: return launch_sgd<7>(s, a, p, stepwise);
        case 8: return launch_sgd<8>(s, a, p, stepwise);
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
    return run_sgd(stream, packed1_dev, packed2_dev, levels_dev, grid_idx_dev, grid_lo, grid_step,
                   grid_max, b_dev, n, d, bits, x_dev, batch, lr, grad_bits, model_bits, seed, epoch,
                   flags, 0, steps, nullptr, nullptr, nullptr, nullptr, nullptr, workspace_dev,
                   workspace_bytes);
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
    return run_sgd(stream, packed1_dev, packed2_dev, levels_dev, grid_idx_dev, grid_lo, grid_step,
                   grid_max, b_dev, n, d, bits, x_dev, batch, lr, grad_bits, model_bits, seed, epoch,
                   flags, step, 1, model_codes_dev, acc_dev, r_dev, g_dev, grad_codes_dev,
                   workspace_dev, workspace_bytes);
}

extern "C" int zipml_sgd_status(void *stream, const void *workspace_dev, size_t workspace_bytes)
{
    if (!workspace_dev || workspace_bytes < 4096) return ZIPML_EWORKSPACE;
    int st = 0;
    hipStream_t s = entry_stream(stream);
    if (hipMemcpyAsync(&st, (const unsigned char *)workspace_dev + Workspace::kStatus, sizeof(int),
                       hipMemcpyDeviceToHost, s) != hipSuccess)
        return ZIPML_ELAUNCH;
    if (hipStreamSynchronize(s) != hipSuccess) return ZIPML_ELAUNCH;
    return st;
}
