// zipml_loss: F(x) = 1/(2n) sum_i (a_i^T x - b_i)^2  (Sec. 1 eq. (1) with the square loss; Sec. 2).
//
// Streaming, sync-free kernels: every workgroup reduces a range of samples to one fp64 partial,
// a second one-block kernel adds the partials in a fixed order.
#include "zipml_device.h"
#include "zipml_host.h"

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
__global__ __launch_bounds__(kLossThreads) void k_loss_copy2(
    const uint32_t *__restrict__ p2, const float *__restrict__ levels, const float *__restrict__ b,
    const float *__restrict__ x, int64_t n, int64_t d, int64_t n_pad, int64_t d32,
    double *__restrict__ partial)
{
    constexpr int K = 1 << BITS;
    __shared__ double scratch[kLossThreads / kWave + 1];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * kLossThreads + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * kLossThreads) {
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
    const double tot = block_sum<double>(acc, scratch);
    if (threadIdx.x == 0) partial[blockIdx.x] = tot;
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

}  // namespace zipml

using namespace zipml;

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
        if (copy == 2) {
            blocks = (int)((n + kLossThreads - 1) / kLossThreads);
            if (blocks > kLossMaxBlocks) blocks = kLossMaxBlocks;
        } else {
            blocks = (int)(lay.n32 > kLossMaxBlocks ? kLossMaxBlocks : lay.n32);
        }
        switch (bits) {
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
