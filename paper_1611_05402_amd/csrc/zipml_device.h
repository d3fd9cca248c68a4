// Device-side building blocks shared by the libzipml kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace zipml {

constexpr int kWave = 64;
constexpr int kGroup = 32;   // features (copy 2) or samples (copy 1) per packed unit

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  Key = seed; counter = (row lo, row hi, col/4,
// epoch*256 + stream).  Word col%4 of the block is the draw of that column.
// ---------------------------------------------------------------------------------------------
struct Philox4 {
    uint32_t w[4];
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        // one 32x32->64 multiply per product (v_mad_u64_u32) instead of separate high and low halves
        const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox4{{c0, c1, c2, c3}};
}

__device__ __forceinline__ Philox4 philox_block(uint64_t seed, uint32_t epoch, uint64_t row,
                                                uint32_t col4, uint32_t stream)
{
    return philox4x32_10((uint32_t)row, (uint32_t)(row >> 32), col4, (epoch << 8) | stream,
                         (uint32_t)seed, (uint32_t)(seed >> 32));
}

// Word k (0..3) of a block, chosen at run time without indexing the register array.
__device__ __forceinline__ uint32_t philox_word(const Philox4 &r, uint32_t k)
{
    return k == 0 ? r.w[0] : k == 1 ? r.w[1] : k == 2 ? r.w[2] : r.w[3];
}

// Top 24 bits as a uniform in [0, 1); exact in fp32.
__device__ __forceinline__ float u24(uint32_t word)
{
    return (float)(word >> 8) * (1.0f / 16777216.0f);
}

// ---------------------------------------------------------------------------------------------
// Packed units: 32 codes of BITS bits each, little-endian bit string in BITS dwords.
// ---------------------------------------------------------------------------------------------
template <int BITS>
__device__ __forceinline__ uint32_t unit_code(const uint32_t (&w)[BITS], int k)
{
    const int bit = k * BITS, wi = bit >> 5, sh = bit & 31;
    uint32_t v = w[wi] >> sh;
    if (sh + BITS > 32) v |= w[wi + 1] << (32 - sh);   // the branch folds: k is a constant after unrolling
    return v & ((1u << BITS) - 1u);
}

template <int BITS>
__device__ __forceinline__ void unit_set(uint32_t (&w)[BITS], int k, uint32_t code)
{
    const int bit = k * BITS, wi = bit >> 5, sh = bit & 31;
    w[wi] |= code << sh;
    if (sh + BITS > 32) w[wi + 1] |= code >> (32 - sh);
}
// (the same on an array of N dwords that holds fewer than 32 codes of `bits` bits)
template <int N>
__device__ __forceinline__ void unit_set(uint32_t (&w)[N], int k, int bits, uint32_t code)
{
    const int bit = k * bits, wi = bit >> 5, sh = bit & 31;
    w[wi] |= code << sh;
    if (sh + bits > 32) w[wi + 1] |= code >> (32 - sh);
}

// A unit from one of its halves: `half` holds sixteen codes as a bit string of 16 BITS bits from bit 0
// (built with unit_set on an array of kHalfDwords dwords, every index a constant); the result is that
// string at bit 0 (h == 0) or at bit 16 BITS (h == 1: BITS / 2 dwords further on, and for odd BITS
// another 16 bits), zeros elsewhere, with every register index still a constant.
template <int BITS> constexpr int kHalfDwords = (16 * BITS + 31) / 32;
template <int BITS>
__device__ __forceinline__ void place_half(uint32_t (&unit)[BITS], const uint32_t (&half)[kHalfDwords<BITS>], int h)
{
    constexpr int HB = kHalfDwords<BITS>, OFF = BITS / 2;
#pragma unroll
    for (int q = 0; q < BITS; ++q) {
        const uint32_t lo = q < HB ? half[q] : 0u;
        uint32_t hi = 0u;
        if constexpr (BITS % 2 == 0) {
            if (q >= OFF && q - OFF < HB) hi = half[q - OFF < HB ? q - OFF : 0];
        } else {
            if (q >= OFF && q - OFF < HB) hi = half[q - OFF < HB ? q - OFF : 0] << 16;
            if (q >= OFF + 1 && q - OFF - 1 < HB) hi |= half[q - OFF - 1 < HB ? q - OFF - 1 : 0] >> 16;
        }
        unit[q] = h ? hi : lo;
    }
}

// ---------------------------------------------------------------------------------------------
// Device-scope (all XCDs) access to data that other workgroups write during the same kernel.
// Each XCD has its own L2, so such data must go through device-coherent accesses.
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ T load_dev(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void store_dev(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void add_dev(T *p, T v)
{
    (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void release_dev()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load, store and atomic of the wave (s_waitcnt vmcnt(0)), which would stall a wave on the
// prefetch it has just issued; this one waits for LDS operations (lgkmcnt) and nothing else.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---------------------------------------------------------------------------------------------
// Wave and block reductions.
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ T wave_sum(T v)
{
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Reductions over lanes with DPP row operations (no LDS traffic); 32-bit types, commutative op.
// Steps: xor 1, xor 2 inside each quad, mirror inside each half row, mirror inside each row of 16.
template <int CTRL, typename T>
__device__ __forceinline__ T dpp_move(T x)
{
    static_assert(sizeof(T) == 4, "32-bit types only");
    int xi = __builtin_bit_cast(int, x);
    xi = __builtin_amdgcn_update_dpp(0, xi, CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(T, xi);
}
// Every lane gets the result over its row of 16 lanes.
template <typename T, typename Op>
__device__ __forceinline__ T row_reduce_dpp(T v, Op op)
{
    v = op(v, dpp_move<0xB1>(v));    // quad_perm [1,0,3,2]
    v = op(v, dpp_move<0x4E>(v));    // quad_perm [2,3,0,1]
    v = op(v, dpp_move<0x141>(v));   // row_half_mirror
    v = op(v, dpp_move<0x140>(v));   // row_mirror
    return v;
}
// Every lane gets the result over the 64 lanes: the four row results are combined through scalar
// registers.
template <typename T, typename Op>
__device__ __forceinline__ T wave_reduce_dpp(T v, Op op)
{
    v = row_reduce_dpp(v, op);
    const int vi = __builtin_bit_cast(int, v);
    const T r0 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(vi, 0));
    const T r1 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(vi, 16));
    const T r2 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(vi, 32));
    const T r3 = __builtin_bit_cast(T, __builtin_amdgcn_readlane(vi, 48));
    return op(op(r0, r1), op(r2, r3));
}
template <typename T>
__device__ __forceinline__ T wave_sum_dpp(T v)
{
    return wave_reduce_dpp(v, [](T x, T y) { return x + y; });
}

// Sum over the block; every thread gets the result.  scratch: >= blockDim/64 + 1 elements of T.
template <typename T>
__device__ __forceinline__ T block_sum(T v, T *scratch)
{
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int nw = (blockDim.x + kWave - 1) >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) scratch[wave] = v;
    __syncthreads();
    T tot = 0;
    for (int w = 0; w < nw; ++w) tot += scratch[w];
    return tot;
}

}  // namespace zipml
