// zipml_quantize / zipml_unpack_codes: fp32 rows -> two independent packed b-bit copies.
//
// Stochastic quantisation of Sec. 2.1 with per-feature levels (Supp. A.3 "Column Scaling") and the
// two independent copies of Sec. 2.2.  One workgroup handles a tile of 32 samples x 128 features:
// it reads the fp32 tile with coalesced 512-byte row segments, takes the rounding decision for both
// copies (one Philox block per copy covers 4 neighbouring features), transposes the codes through
// LDS and writes sample-major units for copy 2 and feature-major units for copy 1.
#include <type_traits>
#include "zipml_device.h"
#include "zipml_host.h"

namespace zipml {

// Bracketing of a value by two neighbouring levels: l = largest c <= K-2 with L[c] <= v (v clamped
// to the level range), and the probability of rounding up to L[l+1] from three correctly rounded
// fp32 operations.
// The index is first guessed from the ends of the table, as if the levels were evenly spaced, and
// then checked against the table itself (L[l] <= v, and l == K-2 or L[l+1] > v: for a
// non-decreasing table that is the definition).  Evenly spaced tables pass at once or after one
// step to a neighbour; any other table falls back to a binary search.  The two table probes are
// branch-free so that the loads of the four elements a thread handles together overlap.
struct Column {
    const float *L;      // levels of this feature
    float L0, Lk, scale; // ends of the table, (K-1) / (Lk - L0) or 0
};
__device__ __forceinline__ Column make_column(const float *__restrict__ L, int K)
{
    Column c;
    c.L = L;
    c.L0 = L[0];
    c.Lk = L[K - 1];
    const float span = c.Lk - c.L0;
    c.scale = span > 0.0f ? __fdividef((float)(K - 1), span) : 0.0f;
    return c;
}
__device__ __forceinline__ bool bracket_ok(int l, int K, float base, float next, float v)
{
    return base <= v && (l == K - 2 || next > v);
}
// Two neighbouring levels with one 8-byte load (4-byte aligned).
typedef float pair_f32 __attribute__((ext_vector_type(2), aligned(4)));
__device__ __forceinline__ void load_pair(const float *__restrict__ p, float &lo, float &hi)
{
    const pair_f32 v = *reinterpret_cast<const pair_f32 *>(p);
    lo = v.x;
    hi = v.y;
}
// Four elements at once; live[e] == false: the element does not exist (l = 0, frac = 0).
// Table probes are gathers (every lane reads another feature's table), which the compute unit
// serves at about one lane per cycle: one 8-byte probe per element, and the second probe only for
// waves in which some lane's guess was off.
__device__ __forceinline__ void bracket4(const Column (&col)[4], const bool (&live)[4], int K,
                                         const float (&vin)[4], int (&l)[4], float (&frac)[4])
{
    float v[4], base[4], next[4];
    bool ok[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[e] = fminf(fmaxf(vin[e], col[e].L0), col[e].Lk);
        int g = (int)((v[e] - col[e].L0) * col[e].scale);
        l[e] = g < 0 ? 0 : g > K - 2 ? K - 2 : g;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        base[e] = next[e] = 0.0f;
        if (live[e]) load_pair(col[e].L + l[e], base[e], next[e]);
    }
    bool all_ok = true;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        ok[e] = !live[e] || bracket_ok(l[e], K, base[e], next[e], v[e]);
        all_ok = all_ok && ok[e];
    }
    if (__any(!all_ok)) {
        // one step towards the value, then the check again; whatever still fails is searched for
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int g = ok[e] ? l[e] : (base[e] > v[e] ? l[e] - 1 : l[e] + 1);
            l[e] = g < 0 ? 0 : g > K - 2 ? K - 2 : g;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (live[e]) load_pair(col[e].L + l[e], base[e], next[e]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (live[e] && !bracket_ok(l[e], K, base[e], next[e], v[e])) {
                int b = 0;
                for (int s = K >> 1; s >= 1; s >>= 1) {
                    const int c = b + s;
                    if (c <= K - 2 && col[e].L[c] <= v[e]) b = c;
                }
                l[e] = b;
                load_pair(col[e].L + b, base[e], next[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float w = next[e] - base[e];
        const float num = v[e] - base[e];
        frac[e] = (live[e] && w > 0.0f) ? __fdiv_rn(num, w) : 0.0f;
        if (!live[e]) l[e] = 0;
    }
}

// One packed unit (BITS contiguous dwords) to global memory, with the widest stores its alignment
// (the largest power of two dividing 4*BITS bytes, at most 16) allows.
template <int BITS>
__device__ __forceinline__ void store_unit(uint32_t *__restrict__ p, const uint32_t (&u)[BITS])
{
    constexpr int kAlign = (BITS % 4 == 0) ? 16 : (BITS % 2 == 0) ? 8 : 4;
    uint32_t *q = static_cast<uint32_t *>(__builtin_assume_aligned(p, kAlign));
#pragma unroll
    for (int k = 0; k < BITS; ++k) q[k] = u[k];
}

constexpr int kTileCols = 64;    // 2 feature groups per workgroup
constexpr int kLdsRow = 17;      // dwords per LDS row of 64 code bytes (+1: conflict-free columns)

// Level tables of the workgroup's 64 features live in LDS ([64][K] floats, staged once); the
// workgroup then walks down its share of the sample groups, 32 samples x 64 features per round
// and 256 threads, with the fp32 values of the next round requested before the current one is
// worked on.  HALVES = 2: two such sets of 256 threads share the tables and take every other
// sample group each -- at 8 bits the 64 KiB of tables leave room for two workgroups per compute
// unit, and with 256 threads each that is two waves per SIMD to hide anything with.
template <int BITS, int HALVES>
__global__ __launch_bounds__(256 * HALVES) void k_quantize_pack(
    const float *__restrict__ A, int64_t n_rows, int64_t d, int64_t lda, int64_t row0,
    int64_t nb64, int64_t n32, int64_t d32, const float *__restrict__ levels, uint64_t seed,
    uint32_t epoch, uint32_t *__restrict__ p1, uint32_t *__restrict__ p2, int vec_ok,
    int64_t groups_per_block, int swapped)
{
    extern __shared__ __align__(16) float tab[];          // [kTileCols][K]
    __shared__ uint32_t c1w_all[HALVES][32 * kLdsRow];
    __shared__ uint32_t c2w_all[HALVES][32 * kLdsRow];
    constexpr int K = 1 << BITS;
    const int hw = HALVES == 1 ? 0 : (int)threadIdx.x >> 8;     // which set of 256 threads
    const int tid = threadIdx.x & 255;                          // thread of the set
    uint32_t *const c1w = c1w_all[hw], *const c2w = c2w_all[hw];
    const int64_t col0 = (int64_t)blockIdx.y * kTileCols;
    for (int e = threadIdx.x; e < kTileCols * K; e += 256 * HALVES) {
        const int64_t j = col0 + e / K;
        tab[e] = j < d ? levels[j * K + e % K] : 0.0f;
    }
    __syncthreads();

    const int cq = tid & 15;                  // which 4 features of the 64
    const int64_t col = col0 + 4 * cq;
    Column cols[4];
    bool live_col[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        live_col[e] = col + e < d;
        cols[e] = make_column(tab + (4 * cq + e) * K, K);
    }
    const int64_t total_groups = (n_rows + 31) / 32;
    const int64_t g_begin = (int64_t)blockIdx.x * groups_per_block;
    const int64_t g_end = g_begin + groups_per_block < total_groups ? g_begin + groups_per_block : total_groups;
    // The loop below exists twice: for workgroups all of whose threads fetch four features with one
    // 16-byte load, and for the others (the last block of features, unaligned rows).  The fetches are
    // loads that no branch can skip -- rows and features past the end repeat the last ones and are
    // never used -- because a load behind a branch makes the compiler wait for every load in flight
    // where the first value is used, the next round's included, and that undoes the prefetch.
    auto run = [&](auto vec_tag) __attribute__((always_inline)) {
    constexpr bool VEC = decltype(vec_tag)::value;
    auto fetch = [&](int64_t rg_local, float (&v)[2][4]) __attribute__((always_inline)) {
        const int64_t rgc = rg_local < g_end ? rg_local : g_end - 1;
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int64_t i = rgc * 32 + pass * 16 + (tid >> 4);
            const float *src = A + (i < n_rows ? i : n_rows - 1) * lda;
            if constexpr (VEC) {
                const float4 q = *reinterpret_cast<const float4 *>(src + col);
                v[pass][0] = q.x; v[pass][1] = q.y; v[pass][2] = q.z; v[pass][3] = q.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[pass][e] = src[col + e < d ? col + e : d - 1];
            }
        }
    };
    // (both sets run the same number of rounds, for the barriers; a set without a group in the last
    // round repeats the loads of the last group and stores nothing)
    float vcur[2][4], vnxt[2][4];
    fetch(g_begin + hw, vcur);
    for (int64_t rg_first = g_begin; rg_first < g_end; rg_first += HALVES) {
        const int64_t rg_local = rg_first + hw;
        const bool active = rg_local < g_end;
        fetch(rg_local + HALVES, vnxt);
        // ---- phase 1: decide both codes of every element of the tile
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int r = pass * 16 + (tid >> 4);
            const int64_t i = rg_local * 32 + r;
            uint32_t w1 = 0, w2 = 0;
            if (active && i < n_rows && col < d) {
                const uint64_t row = (uint64_t)(row0 + i);
                // swapped: the feature-major array gets copy 2 (stream 2), the sample-major copy 1
                const Philox4 r1 = philox_block(seed, epoch, row, (uint32_t)(col >> 2), swapped ? 2u : 1u);
                const Philox4 r2 = philox_block(seed, epoch, row, (uint32_t)(col >> 2), swapped ? 1u : 2u);
                int l[4];
                float frac[4];
                bracket4(cols, live_col, K, vcur[pass], l, frac);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (live_col[e]) {
                        const uint32_t a = (uint32_t)l[e] + (u24(r1.w[e]) < frac[e] ? 1u : 0u);
                        const uint32_t b = (uint32_t)l[e] + (u24(r2.w[e]) < frac[e] ? 1u : 0u);
                        w1 |= a << (8 * e);
                        w2 |= b << (8 * e);
                    }
                }
            }
            c1w[r * kLdsRow + cq] = w1;
            c2w[r * kLdsRow + cq] = w2;
        }
        __syncthreads();

        // ---- phase 2: pack 32 codes per unit and store.  Two neighbouring lanes share a unit, sixteen
        // codes each (with one lane per unit half the workgroup packed while the other half waited
        // at the barrier); the halves are put together with a lane exchange and the even lane stores.
        const int64_t rg = row0 / 32 + rg_local;          // sample group in the whole matrix
        {
            const bool second = tid >= 128;               // waves 0-1: copy 2, waves 2-3: copy 1
            const int u = (tid & 127) >> 1, h = tid & 1;  // unit of the tile, half of the unit
            const int gq = u >> 5, in = u & 31;           // feature group of the tile; sample (copy 2) or feature (copy 1) in it
            const int64_t g = col0 / 32 + gq;
            uint32_t half[kHalfDwords<BITS>];
#pragma unroll
            for (int q = 0; q < kHalfDwords<BITS>; ++q) half[q] = 0;
            if (!second) {
                // copy 2: one unit = sample `in`, feature group gq; this lane's codes 16 h .. 16 h + 15
                // are four words of the tile's row
#pragma unroll
                for (int kk = 0; kk < 16; ++kk) {
                    const uint32_t w = c2w[in * kLdsRow + gq * 8 + 4 * h + (kk >> 2)];
                    unit_set<kHalfDwords<BITS>>(half, kk, BITS, (w >> (8 * (kk & 3))) & 0xFFu);
                }
            } else {
                // copy 1: one unit = feature u of the tile, the 32 samples of this group
#pragma unroll
                for (int kk = 0; kk < 16; ++kk) {
                    const uint32_t w = c1w[(16 * h + kk) * kLdsRow + (u >> 2)];
                    unit_set<kHalfDwords<BITS>>(half, kk, BITS, (w >> (8 * (u & 3))) & 0xFFu);
                }
            }
            uint32_t unit[BITS];
            place_half<BITS>(unit, half, h);
#pragma unroll
            for (int q = 0; q < BITS; ++q) unit[q] |= __shfl_xor(unit[q], 1, 64);
            if (active && h == 0 && g < d32) {
                if (!second) {
                    const int64_t i = rg * 32 + in;
                    store_unit<BITS>(p2 + (g * nb64 * 64 + i) * BITS, unit);
                } else {
                    store_unit<BITS>(p1 + ((g * n32 + rg) * 32 + in) * BITS, unit);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int pass = 0; pass < 2; ++pass)
#pragma unroll
            for (int e = 0; e < 4; ++e) vcur[pass][e] = vnxt[pass][e];
    }
    };
    if (vec_ok && col0 + kTileCols <= d) run(std::true_type{});
    else run(std::false_type{});
}

template <int BITS>
__global__ __launch_bounds__(256) void k_unpack(const uint32_t *__restrict__ packed, int copy,
                                                int64_t n, int64_t d, int64_t n_pad, int64_t n32,
                                                int64_t d32, uint8_t *__restrict__ codes)
{
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // unit index
    if (u >= d32 * n_pad) return;
    uint32_t unit[BITS];
    if (copy == 2) {
        const int64_t g = u / n_pad, i = u % n_pad;
        if (i >= n) return;
        const uint32_t *src = packed + (g * n_pad + i) * BITS;
#pragma unroll
        for (int q = 0; q < BITS; ++q) unit[q] = src[q];
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const int64_t j = g * 32 + k;
            if (j < d) codes[i * d + j] = (uint8_t)unit_code<BITS>(unit, k);
        }
    } else {
        const int64_t g = u / n_pad, rem = u % n_pad, rg = rem / 32, cin = rem % 32;
        const int64_t j = g * 32 + cin;
        if (j >= d) return;
        const uint32_t *src = packed + ((g * n32 + rg) * 32 + cin) * BITS;
#pragma unroll
        for (int q = 0; q < BITS; ++q) unit[q] = src[q];
#pragma unroll
        for (int k = 0; k < 32; ++k) {
            const int64_t i = rg * 32 + k;
            if (i < n) codes[i * d + j] = (uint8_t)unit_code<BITS>(unit, k);
        }
    }
}

// Compact storage of two copies that are stored in the same layout (Sec. 2.2, "Overhead of
// Storing Samples"): the two samples of a value differ by at most one level, so a base level and
// one bit per sample hold both, b + 2 bits per value instead of 2 b.  One thread per packed unit
// of 32 codes.  The record is two planes: the base levels (min of the two codes) as a packed array
// in the layout of the copies, then per unit a pair of dwords of bits (copy a sits one above the
// base; copy b does).  In planes because a kernel that streams the record reads the bases and the
// bits with different instructions: in one interleaved array every memory line would be touched
// by both, and streaming (non-temporal) loads then fetch it twice.  Pairs of codes further apart
// than one level cannot be stored: counted in *bad.
template <int BITS>
__global__ __launch_bounds__(256) void k_compact_encode(const uint32_t *__restrict__ pa,
                                                        const uint32_t *__restrict__ pb, int64_t units,
                                                        uint32_t *__restrict__ out, int *__restrict__ bad)
{
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    uint32_t a[BITS], b[BITS], base[BITS];
#pragma unroll
    for (int q = 0; q < BITS; ++q) { a[q] = pa[u * BITS + q]; b[q] = pb[u * BITS + q]; base[q] = 0u; }
    uint32_t ua = 0u, ub = 0u;
    int wrong = 0;
#pragma unroll
    for (int k = 0; k < 32; ++k) {
        const uint32_t ca = unit_code<BITS>(a, k), cb = unit_code<BITS>(b, k);
        const uint32_t lo = ca < cb ? ca : cb;
        wrong |= (ca - lo > 1u) | (cb - lo > 1u);
        unit_set<BITS>(base, k, lo);
        ua |= ((ca - lo) & 1u) << k;
        ub |= ((cb - lo) & 1u) << k;
    }
    uint32_t *dst = out + u * BITS;
#pragma unroll
    for (int q = 0; q < BITS; ++q) dst[q] = base[q];
    uint32_t *pair = out + units * BITS + 2 * u;
    pair[0] = ua;
    pair[1] = ub;
    if (wrong) atomicAdd(bad, 1);
}

template <int BITS>
__global__ __launch_bounds__(256) void k_compact_decode(const uint32_t *__restrict__ in, int64_t units,
                                                        uint32_t *__restrict__ pa, uint32_t *__restrict__ pb)
{
    const int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= units) return;
    const uint32_t *src = in + u * BITS;
    uint32_t base[BITS], a[BITS], b[BITS];
#pragma unroll
    for (int q = 0; q < BITS; ++q) { base[q] = src[q]; a[q] = 0u; b[q] = 0u; }
    const uint32_t ua = in[units * BITS + 2 * u], ub = in[units * BITS + 2 * u + 1];
#pragma unroll
    for (int k = 0; k < 32; ++k) {
        const uint32_t lo = unit_code<BITS>(base, k);
        unit_set<BITS>(a, k, (lo + ((ua >> k) & 1u)) & ((1u << BITS) - 1u));
        unit_set<BITS>(b, k, (lo + ((ub >> k) & 1u)) & ((1u << BITS) - 1u));
    }
#pragma unroll
    for (int q = 0; q < BITS; ++q) { pa[u * BITS + q] = a[q]; pb[u * BITS + q] = b[q]; }
}

template <int BITS>
static int launch_compact(hipStream_t s, bool encode, const uint32_t *a, const uint32_t *b, int64_t units,
                          uint32_t *compact, uint32_t *oa, uint32_t *ob, int *bad)
{
    const unsigned blocks = (unsigned)((units + 255) / 256);
    if (encode)
        hipLaunchKernelGGL(k_compact_encode<BITS>, dim3(blocks), dim3(256), 0, s, a, b, units, compact, bad);
    else
        hipLaunchKernelGGL(k_compact_decode<BITS>, dim3(blocks), dim3(256), 0, s, compact, units, oa, ob);
    return hip_check(hipGetLastError());
}

template <int BITS>
static int launch_quantize(hipStream_t s, const float *A, int64_t n_rows, int64_t d, int64_t lda,
                           int64_t row0, const Layout &lay, const float *levels, uint64_t seed,
                           uint32_t epoch, uint32_t *p1, uint32_t *p2, int swapped)
{
    const int vec_ok = (lda % 4 == 0) && aligned16(A);
    const int64_t col_blocks = (lay.d + kTileCols - 1) / kTileCols;
    const int64_t groups = (n_rows + 31) / 32;
    // about 2048 workgroups in all, each with at least 4 sample groups to amortise its tables
    int64_t row_blocks = (2048 + col_blocks - 1) / col_blocks;
    if (row_blocks > (groups + 3) / 4) row_blocks = (groups + 3) / 4;
    if (row_blocks < 1) row_blocks = 1;
    if (col_blocks > 65535 || row_blocks > 0x7FFFFFFF) return ZIPML_EUNSUPPORTED;
    const int64_t per_block = (groups + row_blocks - 1) / row_blocks;
    const size_t shmem = (size_t)kTileCols * (1u << BITS) * sizeof(float);
    // (two sets of threads per workgroup where the tables limit the workgroups per compute unit)
    constexpr int kHalves = BITS >= 8 ? 2 : 1;
    if (HIP_FAILED(hipFuncSetAttribute((const void *)k_quantize_pack<BITS, kHalves>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem)))
        return ZIPML_ELAUNCH;
    dim3 grid((unsigned)row_blocks, (unsigned)col_blocks);
    hipLaunchKernelGGL((k_quantize_pack<BITS, kHalves>), grid, dim3(256 * kHalves), shmem, s, A, n_rows, d, lda, row0,
                       lay.nb64, lay.n32, lay.d32, levels, seed, epoch, p1, p2, vec_ok, per_block,
                       swapped);
    return hip_check(hipGetLastError());
}

template <int BITS>
static int launch_unpack(hipStream_t s, const uint32_t *packed, int copy, const Layout &lay,
                         uint8_t *codes)
{
    const int64_t units = lay.d32 * lay.n_pad;
    hipLaunchKernelGGL(k_unpack<BITS>, dim3((unsigned)((units + 255) / 256)), dim3(256), 0, s,
                       packed, copy, lay.n, lay.d, lay.n_pad, lay.n32, lay.d32, codes);
    return hip_check(hipGetLastError());
}

}  // namespace zipml

using namespace zipml;

#define ZIPML_DISPATCH_BITS(bits, CALL)                                           \
    switch (bits) {                                                               \
        case 1: return CALL(1); case 2: return CALL(2); case 3: return CALL(3);   \
        case 4: return CALL(4); case 5: return CALL(5); case 6: return CALL(6);   \
        case 7: return CALL(7); case 8: return CALL(8);                           \
        default: return ZIPML_EINVAL;                                             \
    }

extern "C" size_t zipml_packed_bytes(int64_t n, int64_t d, int bits)
{
    if (n <= 0 || d <= 0 || !valid_bits(bits)) return 0;
    return make_layout(n, d, bits).bytes();
}

static int quantize_entry(void *stream, const float *A_dev, int64_t n_rows, int64_t d, int64_t lda,
                          int64_t row0, int64_t n_total, const float *levels_dev, int bits,
                          uint64_t seed, uint32_t epoch, void *packed1_dev, void *packed2_dev,
                          int swapped)
{
    if (!A_dev || !levels_dev || !packed1_dev || !packed2_dev) return ZIPML_EINVAL;
    if (n_rows <= 0 || d <= 0 || lda < d || n_total <= 0 || !valid_bits(bits)) return ZIPML_EINVAL;
    if (row0 < 0 || row0 % 32 != 0 || row0 + n_rows > n_total) return ZIPML_EINVAL;
    if (n_rows % 32 != 0 && row0 + n_rows != n_total) return ZIPML_EINVAL;
    if (epoch >= (1u << 24)) return ZIPML_EINVAL;
    if (!aligned16(levels_dev) || !aligned16(packed1_dev) || !aligned16(packed2_dev) ||
        (reinterpret_cast<uintptr_t>(A_dev) & 3u))
        return ZIPML_EALIGN;
    const Layout lay = make_layout(n_total, d, bits);
    hipStream_t s = entry_stream(stream);
    uint32_t *p1 = (uint32_t *)packed1_dev, *p2 = (uint32_t *)packed2_dev;
#define CALL(B) launch_quantize<B>(s, A_dev, n_rows, d, lda, row0, lay, levels_dev, seed, epoch, p1, p2, swapped)
    ZIPML_DISPATCH_BITS(bits, CALL)
#undef CALL
}

extern "C" int zipml_quantize(void *stream, const float *A_dev, int64_t n_rows, int64_t d,
                              int64_t lda, int64_t row0, int64_t n_total,
                              const float *levels_dev, int bits, uint64_t seed, uint32_t epoch,
                              void *packed1_dev, void *packed2_dev)
{
    return quantize_entry(stream, A_dev, n_rows, d, lda, row0, n_total, levels_dev, bits, seed, epoch,
                          packed1_dev, packed2_dev, 0);
}

extern "C" int zipml_quantize_swapped(void *stream, const float *A_dev, int64_t n_rows, int64_t d,
                                      int64_t lda, int64_t row0, int64_t n_total,
                                      const float *levels_dev, int bits, uint64_t seed,
                                      uint32_t epoch, void *packed1s_dev, void *packed2s_dev)
{
    return quantize_entry(stream, A_dev, n_rows, d, lda, row0, n_total, levels_dev, bits, seed, epoch,
                          packed1s_dev, packed2s_dev, 1);
}

extern "C" int zipml_unpack_codes(void *stream, const void *packed_dev, int copy, int64_t n,
                                  int64_t d, int bits, uint8_t *codes_dev)
{
    if (!packed_dev || !codes_dev || n <= 0 || d <= 0 || !valid_bits(bits)) return ZIPML_EINVAL;
    if (copy != 1 && copy != 2) return ZIPML_EINVAL;
    if (!aligned16(packed_dev)) return ZIPML_EALIGN;
    const Layout lay = make_layout(n, d, bits);
    hipStream_t s = entry_stream(stream);
#define CALL(B) launch_unpack<B>(s, (const uint32_t *)packed_dev, copy, lay, codes_dev)
    ZIPML_DISPATCH_BITS(bits, CALL)
#undef CALL
}

extern "C" size_t zipml_compact_bytes(int64_t n, int64_t d, int bits)
{
    if (n <= 0 || d <= 0 || !valid_bits(bits)) return 0;
    const Layout lay = make_layout(n, d, bits);
    return (size_t)lay.n_pad * (size_t)lay.d_pad / 32 * (size_t)(bits + 2) * 4;
}

extern "C" int zipml_compact_encode(void *stream, const void *packed_a_dev, const void *packed_b_dev,
                                    int64_t n, int64_t d, int bits, void *compact_dev,
                                    void *workspace_dev, size_t workspace_bytes)
{
    if (!packed_a_dev || !packed_b_dev || !compact_dev || n <= 0 || d <= 0 || !valid_bits(bits))
        return ZIPML_EINVAL;
    if (!workspace_dev || workspace_bytes < 256) return ZIPML_EWORKSPACE;
    if (!aligned16(packed_a_dev) || !aligned16(packed_b_dev) || !aligned16(compact_dev) ||
        !aligned16(workspace_dev))
        return ZIPML_EALIGN;
    const Layout lay = make_layout(n, d, bits);
    const int64_t units = lay.n_pad * lay.d_pad / 32;
    hipStream_t s = entry_stream(stream);
    int *bad = (int *)workspace_dev;
    if (hipMemsetAsync(bad, 0, sizeof(int), s) != hipSuccess) return ZIPML_ELAUNCH;
    int rc = ZIPML_EINVAL;
#define CALL(B) launch_compact<B>(s, true, (const uint32_t *)packed_a_dev, (const uint32_t *)packed_b_dev, \
                                  units, (uint32_t *)compact_dev, nullptr, nullptr, bad)
    switch (bits) {
        case 1: rc = CALL(1); break; case 2: rc = CALL(2); break; case 3: rc = CALL(3); break;
        case 4: rc = CALL(4); break; case 5: rc = CALL(5); break; case 6: rc = CALL(6); break;
        case 7: rc = CALL(7); break; case 8: rc = CALL(8); break;
    }
#undef CALL
    if (rc) return rc;
    int bad_host = 0;
    if (hipMemcpyAsync(&bad_host, bad, sizeof(int), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return ZIPML_ELAUNCH;
    return bad_host ? ZIPML_EINVAL : ZIPML_OK;     // some pair of codes differs by more than one level
}

extern "C" int zipml_compact_decode(void *stream, const void *compact_dev, int64_t n, int64_t d,
                                    int bits, void *packed_a_dev, void *packed_b_dev)
{
    if (!packed_a_dev || !packed_b_dev || !compact_dev || n <= 0 || d <= 0 || !valid_bits(bits))
        return ZIPML_EINVAL;
    if (!aligned16(packed_a_dev) || !aligned16(packed_b_dev) || !aligned16(compact_dev)) return ZIPML_EALIGN;
    const Layout lay = make_layout(n, d, bits);
    const int64_t units = lay.n_pad * lay.d_pad / 32;
    hipStream_t s = entry_stream(stream);
#define CALL(B) launch_compact<B>(s, false, nullptr, nullptr, units, (uint32_t *)const_cast<void *>(compact_dev), \
                                  (uint32_t *)packed_a_dev, (uint32_t *)packed_b_dev, nullptr)
    ZIPML_DISPATCH_BITS(bits, CALL)
#undef CALL
}
