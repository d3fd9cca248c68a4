// Operand helpers of the matrix-core paths (v_mfma_i32_16x16x64_i8 on packed low-bit codes against
// fixed-point digits): shared by the SGD step loops and the loss kernel.
//
// Operand layout of the instruction (checked against a host reference on the device):
//   A: lane l holds row l%16, k = 16*(l/16) .. +15 (16 bytes);  B: lane l holds column l%16, same k;
//   C: lane l holds column l%16, rows 4*(l/16) .. +3.
// A lane's 16 code bytes come from 16*BITS/8 packed bytes; code_slot() says which byte a code of
// the packed unit lands in, and the digit operands are laid out in LDS with the same map.
#pragma once
#include "zipml_device.h"

#include <math.h>

namespace zipml {

typedef int v4i __attribute__((ext_vector_type(4)));

// Code f (0..31) of a packed unit -> (half: which lane operand of 16 codes, byte inside it).
template <int BITS>
__device__ __forceinline__ void code_slot(int f, int &half, int &byte)
{
    if (BITS == 8) {            // 4 dwords per half, code = 16*half + byte
        half = f >> 4;
        byte = f & 15;
    } else if (BITS == 4) {     // packed dword pd holds codes 8pd..8pd+7; low nibbles -> one operand
        const int pd = f >> 3, e = f & 7;    // dword, high nibbles -> the next
        half = pd >> 1;
        byte = (2 * (pd & 1) + (e & 1)) * 4 + (e >> 1);
    } else {                    // BITS == 2: one packed dword per half; operand dword D = (p >> 2D) & 0x03..
        const int e = f & 15;
        half = f >> 4;
        byte = (e & 3) * 4 + (e >> 2);
    }
}

// 16 packed codes (BITS/2 dwords) -> 16 signed bytes (code - off).
template <int BITS>
__device__ __forceinline__ v4i expand_codes(const uint32_t (&p)[BITS / 2])
{
    v4i r;
    if constexpr (BITS == 8) {
        r[0] = (int)(p[0] ^ 0x80808080u);
        r[1] = (int)(p[1] ^ 0x80808080u);
        r[2] = (int)(p[2] ^ 0x80808080u);
        r[3] = (int)(p[3] ^ 0x80808080u);
    } else if constexpr (BITS == 4) {
        r[0] = (int)(p[0] & 0x0F0F0F0Fu);
        r[1] = (int)((p[0] >> 4) & 0x0F0F0F0Fu);
        r[2] = (int)(p[1] & 0x0F0F0F0Fu);
        r[3] = (int)((p[1] >> 4) & 0x0F0F0F0Fu);
    } else {
        r[0] = (int)(p[0] & 0x03030303u);
        r[1] = (int)((p[0] >> 2) & 0x03030303u);
        r[2] = (int)((p[0] >> 4) & 0x03030303u);
        r[3] = (int)((p[0] >> 6) & 0x03030303u);
    }
    return r;
}

// v = d0 + 256 d1 + 65536 d2 + 2^24 d3 with signed bytes d_k (|v| < 2^30): adding 128 to each of
// the three low bytes (carries included) leaves d_k + 128 in byte k, and x + 128 -> x is a flip of
// the top bit.  Returns the four digits as the bytes of one dword.
__device__ __forceinline__ uint32_t signed_digits(int v)
{
    return ((uint32_t)v + 0x00808080u) ^ 0x00808080u;
}
// Digit k of an element goes to plane k: 64 bytes apart.
__device__ __forceinline__ void store_digits(int8_t *plane0, uint32_t dg)
{
    plane0[0] = (int8_t)(dg & 0xFF);
    plane0[64] = (int8_t)((dg >> 8) & 0xFF);
    plane0[128] = (int8_t)((dg >> 16) & 0xFF);
    plane0[192] = (int8_t)(dg >> 24);
}

__device__ __forceinline__ long long combine_digits(const v4i &c)
{
    return (long long)c[0] + ((long long)c[1] << 8) + ((long long)c[2] << 16) + ((long long)c[3] << 24);
}

// int64 (|v| < 2^53) times 2^-k as fp32, rounded once.
__device__ __forceinline__ float fixed_to_float(long long v, int k)
{
    const double d = (double)(int)(v >> 32) * 4294967296.0 + (double)(uint32_t)v;
    return (float)ldexp(d, -k);
}

// Largest k (clamped to +-60) with 2^k * v < 2^bits, for finite v >= 0.
__device__ __forceinline__ int scale_exponent(float v, int bits)
{
    if (!(v > 0.0f)) return 60;
    int e = 0;
    (void)frexpf(v, &e);     // v = m 2^e, 0.5 <= m < 1
    const int k = bits - e;
    return k < -60 ? -60 : k > 60 ? 60 : k;
}

}  // namespace zipml
