// zipml_loss: F(x) = 1/(2n) sum_i (a_i^T x - b_i)^2  (Sec. 1 eq. (1) with the square loss; Sec. 2).
//
// Streaming, sync-free kernels: every workgroup reduces a range of samples to one fp64 partial,
// a second one-block kernel adds the partials in a fixed order.
#include "zipml_device.h"
#include "zipml_host.h"
#include "zipml_mfma_ops.h"

#include <stdlib.h>

namespace zipml {

constexpr int kLossThreads = 256;
constexpr int kLossMaxBlocks = 2048;

// fp32 rows: `lpr` lanes (a power of two <= 64) share one sample and stride over its features.
__global__ __launch_bounds__(kLossThreads) void k_loss_fp32(
    const float *__restrict__ A, int64_t lda, const float *__restrict__ b,
    const float *__restrict__ x, int64_t n, int64_t d, int lpr, int vec_ok,
    double *__restrict__ partial)
{
    __shared__ double scratch[kLossThreads / kWave + 1];
    const int tid = threadIdx.x;
    const int sub = tid % lpr;
    const int64_t rows_per_block = kLossThreads / lpr;
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * rows_per_block + tid / lpr; i < n;
         i += (int64_t)gridDim.x * rows_per_block) {
        const float *row = A + i * lda;
        float z = 0.0f;
        if (vec_ok) {
            for (int64_t j = 4 * sub; j < d; j += 4 * lpr) {
                const float4 av = *reinterpret_cast<const float4 *>(row + j);
                const float4 xv = *reinterpret_cast<const float4 *>(x + j);
                z = fmaf(av.x, xv.x, z);
                z = fmaf(av.y, xv.y, z);
                z = fmaf(av.z, xv.z, z);
                z = fmaf(av.w, xv.w, z);
            }
        } else {
            for (int64_t j = sub; j < d; j += lpr) z = fmaf(row[j], x[j], z);
        }
        for (int off = lpr / 2; off > 0; off >>= 1) z += __shfl_xor(z, off, kWave);
        if (sub == 0) {
            const double r = (double)z - (double)b[i];
            acc += r * r;
        }
    }
    const double tot = block_sum<double>(acc, scratch);
    if (tid == 0) partial[blockIdx.x] = tot;
}

// Packed copy 2 (sample-major units): one sample per thread, feature groups in sequence.
template <int BITS>
__device__ __forceinline__ double loss_copy2_rows(const uint32_t *__restrict__ p2,
                                                  const float *__restrict__ levels,
                                                  const float *__restrict__ b,
                                                  const float *__restrict__ x, int64_t n, int64_t d,
                                                  int64_t n_pad, int64_t d32, int threads)
{
    constexpr int K = 1 << BITS;
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * threads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * threads) {
        float z = 0.0f;
        for (int64_t g = 0; g < d32; ++g) {
            uint32_t u[BITS];
#pragma unroll
            for (int q = 0; q < BITS; ++q) u[q] = p2[(g * n_pad + i) * BITS + q];
#pragma unroll
            for (int k = 0; k < 32; ++k) {
                const int64_t j = g * 32 + k;
                if (j < d) z = fmaf(levels[j * K + unit_code<BITS>(u, k)], x[j], z);
            }
        }
        const double r = (double)z - (double)b[i];
        acc += r * r;
    }
    return acc;
}

template <int BITS>
__global__ __launch_bounds__(kLossThreads) void k_loss_copy2(
    const uint32_t *__restrict__ p2, const float *__restrict__ levels, const float *__restrict__ b,
    const float *__restrict__ x, int64_t n, int64_t d, int64_t n_pad, int64_t d32,
    double *__restrict__ partial)
{
    __shared__ double scratch[kLossThreads / kWave + 1];
    const double acc = loss_copy2_rows<BITS>(p2, levels, b, x, n, d, n_pad, d32, kLossThreads);
    const double tot = block_sum<double>(acc, scratch);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

// Are the level tables evenly spaced (fp64 formula, rounded once)?  One flag per block; K a
// multiple of 4.  (The same test as in the preparation of the SGD kernels.)
constexpr int kLossEvenBlocks = 64;
__global__ __launch_bounds__(256) void k_loss_even(const float *__restrict__ levels, int64_t d, int K,
                                                   int *__restrict__ even)
{
    const int spf = K / 4;
    const int64_t total = d * spf;
    const int64_t per = (total + kLossEvenBlocks - 1) / kLossEvenBlocks;
    const int64_t s_end = (blockIdx.x + 1) * per < total ? (blockIdx.x + 1) * per : total;
    int ok = 1;
    for (int64_t sg = blockIdx.x * per + threadIdx.x; sg < s_end; sg += 256) {
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

// Packed copy 2 with evenly spaced 2-, 4- or 8-bit levels, on the matrix cores: a value is
// mid_j + (code - off) delta_j, so  a_i^T x = sum_j mid_j x_j + sum_j (code_ij - off) y_j  with
// y_j = delta_j x_j.  y goes to 32-bit fixed point in four signed base-256 digits kept in LDS; a
// workgroup takes tiles of 64 samples, its eight waves split the 64-feature blocks (one
// v_mfma_i32_16x16x64_i8 per 16 samples x 64 features, four sample tiles sharing one accumulator
// as in the SGD kernels), the partial sums meet in LDS and wave 0 squares the residuals.  Exact
// integer sums; the only rounding before the residual is y_j -> fixed point (2^-29 of max |y|).
// If the tables turn out not to be evenly spaced (flags from k_loss_even) the kernel takes the
// one-sample-per-thread path above.
constexpr int kLossMfmaThreads = 512;
template <int BITS>
__global__ __launch_bounds__(kLossMfmaThreads) void k_loss_copy2_mfma(
    const uint32_t *__restrict__ p2, const float *__restrict__ levels, const float *__restrict__ b,
    const float *__restrict__ x, int64_t n, int64_t d, int64_t n_pad, int64_t d32, int NKB,
    const int *__restrict__ even, double *__restrict__ partial)
{
    constexpr int K = 1 << BITS, HW = BITS / 2, kW = kLossMfmaThreads / kWave;
    constexpr float kOff = BITS == 8 ? 128.0f : 0.0f;
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ double scratch[kW + 1];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int n16 = lane & 15, q4 = lane >> 4;
    int ok_all = 1;
    if (tid < kLossEvenBlocks) ok_all = even[tid];
    if (!__syncthreads_and(ok_all)) {
        const double acc = loss_copy2_rows<BITS>(p2, levels, b, x, n, d, n_pad, d32, kLossMfmaThreads);
        const double tot = block_sum<double>(acc, scratch);
        if (tid == 0) partial[blockIdx.x] = tot;
        return;
    }
    const int nfeat = NKB * 64;
    int8_t *const ydig = (int8_t *)smem;                                  // [NKB][4 digits][4 q][16]
    float *const ytmp = (float *)(smem + (size_t)NKB * 256);              // [nfeat] y_j until the scale is known
    long long *const zpart = (long long *)(smem + (size_t)NKB * 512);     // [kW][64]
    float *const red = (float *)(smem + (size_t)NKB * 512 + kW * 64 * 8); // [2 kW]
    int8_t *const zeros = (int8_t *)(red + 2 * kW);                       // [16]
    if (tid < 4) reinterpret_cast<int *>(zeros)[tid] = 0;

    // ---- digits of y_j = delta_j x_j and sum_j mid_j x_j (every workgroup: the same numbers)
    float ymax = 0.0f, cqp = 0.0f;
    for (int j = tid; j < nfeat; j += kLossMfmaThreads) {
        float y = 0.0f;
        if (j < d) {
            const float lo = levels[(size_t)j * K], hi = levels[(size_t)j * K + K - 1];
            const float dl = (float)(((double)hi - (double)lo) / (double)(K - 1));
            const float xj = x[j];
            y = dl * xj;
            cqp += (lo + kOff * dl) * xj;
        }
        ymax = fmaxf(ymax, fabsf(y));
        ytmp[j] = y;
    }
    ymax = wave_reduce_dpp(ymax, [](float u, float v) { return fmaxf(u, v); });
    cqp = wave_sum_dpp(cqp);
    if (lane == 0) { red[wave] = ymax; red[kW + wave] = cqp; }
    __syncthreads();
    float cq = 0.0f;
    ymax = 0.0f;
#pragma unroll
    for (int v = 0; v < kW; ++v) { ymax = fmaxf(ymax, red[v]); cq += red[kW + v]; }
    const int ky = scale_exponent(ymax, 29);
    for (int j = tid; j < nfeat; j += kLossMfmaThreads) {
        int half, byte;
        code_slot<BITS>(j & 31, half, byte);
        const int pos = (2 * ((j >> 5) & 1) + half) * 16 + byte;
        store_digits(ydig + (j >> 6) * 256 + pos, signed_digits(__float2int_rn(ldexpf(ytmp[j], ky))));
    }
    __syncthreads();

    // ---- tiles of 64 samples
    const int dig_off = (n16 & 3) * 64 + q4 * 16, slot_of = n16 >> 2;
    const int zero_off = (int)(zeros - ydig);
    const int64_t NT = n_pad / 64;
    double acc = 0.0;
    for (int64_t T = blockIdx.x; T < NT; T += gridDim.x) {
        const int64_t row0 = 64 * T;
        v4i c = {0, 0, 0, 0};
        for (int kb = wave; kb < NKB; kb += kW) {
            // lane = sample 16 sl + n16 of the tile, 16 codes (half q4 & 1) of feature group 2 kb + q4 / 2;
            // a padding group (odd number of groups) reads the block's first group: its digits are zero
            int64_t g = 2 * kb + (q4 >> 1);
            g = g < d32 ? g : 2 * kb;
            uint32_t w[4][HW];
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                const uint32_t *q = static_cast<const uint32_t *>(__builtin_assume_aligned(
                    p2 + (g * n_pad + row0 + 16 * sl + n16) * BITS + (q4 & 1) * HW, 4 * HW));
#pragma unroll
                for (int h = 0; h < HW; ++h) w[sl][h] = __builtin_nontemporal_load(q + h);
            }
#pragma unroll
            for (int sl = 0; sl < 4; ++sl) {
                const v4i ad = *reinterpret_cast<const v4i *>(ydig + (slot_of == sl ? kb * 256 + dig_off : zero_off));
                c = __builtin_amdgcn_mfma_i32_16x16x64_i8(ad, expand_codes<BITS>(w[sl]), c, 0, 0, 0);
            }
        }
        zpart[wave * 64 + lane] = combine_digits(c);      // lane = sample of the tile
        __syncthreads();
        if (wave == 0) {
            long long z = 0;
#pragma unroll
            for (int v = 0; v < kW; ++v) z += zpart[v * 64 + lane];
            if (row0 + lane < n) {
                const double r = ldexp((double)z, -ky) + (double)cq - (double)b[row0 + lane];
                acc += r * r;
            }
        }
        __syncthreads();
    }
    const double tot = block_sum<double>(acc, scratch);
    if (tid == 0) partial[blockIdx.x] = tot;
}

// LDS of k_loss_copy2_mfma.
inline size_t loss_mfma_lds_bytes(int NKB)
{
    return (size_t)NKB * 512 + (kLossMfmaThreads / kWave) * 64 * 8 + 2 * (kLossMfmaThreads / kWave) * 4 + 16;
}

// Packed copy 1 (feature-major units): one workgroup per group of 32 samples; threads stride over
// the features and keep 32 partial dot products each, which are then added across the block.
template <int BITS>
__global__ __launch_bounds__(kLossThreads) void k_loss_copy1(
    const uint32_t *__restrict__ p1, const float *__restrict__ levels, const float *__restrict__ b,
    const float *__restrict__ x, int64_t n, int64_t d, int64_t n32, double *__restrict__ partial)
{
    constexpr int K = 1 << BITS;
    __shared__ float zs[32];
    __shared__ double scratch[kLossThreads / kWave + 1];
    double acc = 0.0;
    for (int64_t rg = blockIdx.x; rg < n32; rg += gridDim.x) {
        float z[32];
#pragma unroll
        for (int k = 0; k < 32; ++k) z[k] = 0.0f;
        for (int64_t j = threadIdx.x; j < d; j += kLossThreads) {
            const int64_t g = j / 32, cin = j % 32;
            uint32_t u[BITS];
#pragma unroll
            for (int q = 0; q < BITS; ++q) u[q] = p1[((g * n32 + rg) * 32 + cin) * BITS + q];
            const float xj = x[j];
#pragma unroll
            for (int k = 0; k < 32; ++k) z[k] = fmaf(levels[j * K + unit_code<BITS>(u, k)], xj, z[k]);
        }
        if (threadIdx.x < 32) zs[threadIdx.x] = 0.0f;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const float s = wave_sum(z[k]);
            if ((threadIdx.x & (kWave - 1)) == 0) atomicAdd(&zs[k], s);
        }
        __syncthreads();
        if (threadIdx.x < 32) {
            const int64_t i = rg * 32 + threadIdx.x;
            if (i < n) {
                const double r = (double)zs[threadIdx.x] - (double)b[i];
                acc += r * r;
            }
        }
        __syncthreads();
    }
    const double tot = block_sum<double>(acc, scratch);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
}

__global__ void k_loss_final(const double *__restrict__ partial, int count, double scale,
                             double *__restrict__ out)
{
    __shared__ double scratch[kLossThreads / kWave + 1];
    double acc = 0.0;
    for (int i = threadIdx.x; i < count; i += blockDim.x) acc += partial[i];
    const double tot = block_sum<double>(acc, scratch);
    if (threadIdx.x == 0) out[0] = tot * scale;
}

template <int BITS>
static void launch_loss_packed(hipStream_t s, const uint32_t *p, int copy, const Layout &lay,
                               const float *levels, const float *b, const float *x, int blocks,
                               double *partial)
{
    if (copy == 2)
        hipLaunchKernelGGL(k_loss_copy2<BITS>, dim3(blocks), dim3(kLossThreads), 0, s, p, levels, b,
                           x, lay.n, lay.d, lay.n_pad, lay.d32, partial);
    else
        hipLaunchKernelGGL(k_loss_copy1<BITS>, dim3(blocks), dim3(kLossThreads), 0, s, p, levels, b,
                           x, lay.n, lay.d, lay.n32, partial);
}

// Copy 2 on the matrix cores where the code width allows it (the kernel itself falls back to the
// one-sample-per-thread path if the tables are not evenly spaced).  Returns the number of blocks,
// 0 if this path does not apply.
template <int BITS>
static int launch_loss_mfma(hipStream_t s, const uint32_t *p, const Layout &lay, const float *levels,
                            const float *b, const float *x, double *partial, int *even, int lds_limit)
{
    const int NKB = (int)((lay.d32 + 1) / 2);
    const size_t shmem = loss_mfma_lds_bytes(NKB);
    if (shmem > (size_t)lds_limit) return 0;
    const void *kern = (const void *)k_loss_copy2_mfma<BITS>;
    if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem) != hipSuccess)
        return 0;
    const int64_t NT = lay.n_pad / 64;
    const int blocks = (int)(NT < 1024 ? NT : 1024);
    hipLaunchKernelGGL(k_loss_even, dim3(kLossEvenBlocks), dim3(256), 0, s, levels, lay.d, 1 << BITS, even);
    hipLaunchKernelGGL(k_loss_copy2_mfma<BITS>, dim3(blocks), dim3(kLossMfmaThreads), shmem, s, p, levels,
                       b, x, lay.n, lay.d, lay.n_pad, lay.d32, NKB, even, partial);
    return blocks;
}

// A plain streaming kernel of known size: reads `n16` 16-byte words once (non-temporal loads, four
// in flight per thread), XORs their dwords into *sink, and, with dst, stores them as well.
__global__ __launch_bounds__(256) void k_stream_probe(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                      size_t n16, uint32_t *sink)
{
    typedef unsigned int u4 __attribute__((ext_vector_type(4)));
    const u4 *in = reinterpret_cast<const u4 *>(src);
    u4 *out = reinterpret_cast<u4 *>(dst);
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    uint32_t x = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = __builtin_nontemporal_load(in + i + k * stride);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (out) __builtin_nontemporal_store(v[k], out + i + k * stride);
            x ^= v[k][0] ^ v[k][1] ^ v[k][2] ^ v[k][3];
        }
    }
    for (; i < n16; i += stride) {
        const u4 v = __builtin_nontemporal_load(in + i);
        if (out) __builtin_nontemporal_store(v, out + i);
        x ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
    x = wave_reduce_dpp(x, [](uint32_t p, uint32_t q) { return p ^ q; });
    if ((threadIdx.x & (kWave - 1)) == 0) atomicXor(sink, x);
}

}  // namespace zipml

using namespace zipml;

extern "C" int zipml_debug_stream(void *stream, const void *src_dev, void *dst_dev, size_t bytes,
                                  uint32_t *sink_dev)
{
    if (!src_dev || !sink_dev || bytes == 0 || bytes % 16 != 0) return ZIPML_EINVAL;
    if (!aligned16(src_dev) || (dst_dev && !aligned16(dst_dev)) || (reinterpret_cast<uintptr_t>(sink_dev) & 3u))
        return ZIPML_EALIGN;
    hipStream_t s = entry_stream(stream);
    const size_t n16 = bytes / 16;
    const size_t want = (n16 + 256 * 4 - 1) / (256 * 4);
    const unsigned blocks = (unsigned)(want < 1 ? 1 : want > 4096 ? 4096 : want);
    hipLaunchKernelGGL(k_stream_probe, dim3(blocks), dim3(256), 0, s, (const uint4 *)src_dev, (uint4 *)dst_dev,
                       n16, sink_dev);
    if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    return ZIPML_OK;
}

extern "C" int zipml_loss(void *stream, const float *A_dev, int64_t lda, const void *packed_dev,
                          int copy, const float *levels_dev, int bits, const float *b_dev,
                          const float *x_dev, int64_t n, int64_t d, double *loss_host,
                          void *workspace_dev, size_t workspace_bytes)
{
    if (!b_dev || !x_dev || !loss_host || n <= 0 || d <= 0) return ZIPML_EINVAL;
    if (!workspace_dev || workspace_bytes < (size_t)(kLossMaxBlocks + 1) * sizeof(double))
        return ZIPML_EWORKSPACE;
    if (!aligned16(workspace_dev) || !aligned16(x_dev)) return ZIPML_EALIGN;
    hipStream_t s = entry_stream(stream);
    double *partial = (double *)workspace_dev;
    double *out = partial + kLossMaxBlocks;
    int blocks = 0;
    if (A_dev) {
        if (lda < d) return ZIPML_EINVAL;
        if (reinterpret_cast<uintptr_t>(A_dev) & 3u) return ZIPML_EALIGN;
        int lpr = 1;
        while (lpr < 64 && lpr * 4 < d) lpr <<= 1;
        const int vec_ok = (lda % 4 == 0) && (d % 4 == 0) && aligned16(A_dev);
        const int64_t rows_per_block = kLossThreads / lpr;
        blocks = (int)((n + rows_per_block - 1) / rows_per_block);
        if (blocks > kLossMaxBlocks) blocks = kLossMaxBlocks;
        hipLaunchKernelGGL(k_loss_fp32, dim3(blocks), dim3(kLossThreads), 0, s, A_dev, lda, b_dev,
                           x_dev, n, d, lpr, vec_ok, partial);
    } else {
        if (!packed_dev || !levels_dev || !valid_bits(bits) || (copy != 1 && copy != 2))
            return ZIPML_EINVAL;
        if (!aligned16(packed_dev) || !aligned16(levels_dev)) return ZIPML_EALIGN;
        const Layout lay = make_layout(n, d, bits);
        const uint32_t *p = (const uint32_t *)packed_dev;
        // copy 2, 2/4/8 bits: matrix-core kernel (needs room for its flags behind the partials)
        const size_t flags_at = (size_t)(kLossMaxBlocks + 1) * sizeof(double);
        if (copy == 2 && (bits == 2 || bits == 4 || bits == 8) &&
            workspace_bytes >= flags_at + kLossEvenBlocks * sizeof(int) && knob(ZIPML_KNOB_NO_MATRIX_CORES) <= 0) {
            int dev = 0, lds = 0;
            if (hipGetDevice(&dev) == hipSuccess &&
                hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess) {
                int *even = (int *)((unsigned char *)workspace_dev + flags_at);
                blocks = bits == 2 ? launch_loss_mfma<2>(s, p, lay, levels_dev, b_dev, x_dev, partial, even, lds)
                       : bits == 4 ? launch_loss_mfma<4>(s, p, lay, levels_dev, b_dev, x_dev, partial, even, lds)
                                   : launch_loss_mfma<8>(s, p, lay, levels_dev, b_dev, x_dev, partial, even, lds);
            }
        }
        const bool launched = blocks > 0;
        if (launched) {
            // (the matrix-core kernel has been launched above)
        } else if (copy == 2) {
            blocks = (int)((n + kLossThreads - 1) / kLossThreads);
            if (blocks > kLossMaxBlocks) blocks = kLossMaxBlocks;
        } else {
            blocks = (int)(lay.n32 > kLossMaxBlocks ? kLossMaxBlocks : lay.n32);
        }
        if (!launched) switch (bits) {
            case 1: launch_loss_packed<1>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
            case 2: launch_loss_packed<2>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
            case 3: launch_loss_packed<3>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
            case 4: launch_loss_packed<4>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
            case 5: launch_loss_packed<5>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
            case 6: launch_loss_packed<6>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
            case 7: launch_loss_packed<7>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
            case 8: launch_loss_packed<8>(s, p, copy, lay, levels_dev, b_dev, x_dev, blocks, partial); break;
        }
    }
    if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    hipLaunchKernelGGL(k_loss_final, dim3(1), dim3(kLossThreads), 0, s, partial, blocks,
                       1.0 / (2.0 * (double)n), out);
    if (HIP_FAILED(hipGetLastError())) return ZIPML_ELAUNCH;
    if (hipMemcpyAsync(loss_host, out, sizeof(double), hipMemcpyDeviceToHost, s) != hipSuccess)
        return ZIPML_ELAUNCH;
    if (hipStreamSynchronize(s) != hipSuccess) return ZIPML_ELAUNCH;
    return ZIPML_OK;
}
