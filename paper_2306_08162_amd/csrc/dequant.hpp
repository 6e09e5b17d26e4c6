// In-register dequantisation of packed codes to 16-bit MFMA operands (Sec. 3.1 "standard unpacking",
// grouped affine form s * (q - z)).
//
// A thread always holds one "unit": 32 consecutive codes of one weight row = BITS 32-bit words, all in one
// quantisation group (group sizes are multiples of 32).  dequant8<BITS,BF16>(w, part, c) returns codes
// [8*part, 8*part+8) of the unit, in k order, as eight 16-bit floats, each rounded once from the exact product.
//
// fp16: a code is dropped into the mantissa of the constant 1024.0 (bits 0x6400), giving 1024 + c * 2^p exactly
// for a code sitting at bit p of a 16-bit lane; one packed fma with (2^-p, -(1024 * 2^-p + z)) yields the exact
// small integer c - z, and one packed multiply applies the scale.  bf16: there is no packed bf16 arithmetic, so
// codes go through fp32 (fma(c, s, -z s)) and are packed with the hardware bf16 conversion.
#pragma once
#include "common.hpp"

namespace qlora {

template <int BITS, bool BF16>
struct DequantConst;

template <int BITS>
struct DequantConst<BITS, false> {
    half2_t s2;        // (s, s)
    half2_t off[2];    // additive constants per code-pair pattern
    __device__ __forceinline__ void set(float s, float z)
    {
        s2 = half2_t{(half_t)s, (half_t)s};
        if constexpr (BITS == 4) {
            off[0] = half2_t{(half_t)(-(1024.f + z)), (half_t)(-(64.f + z))};
        } else if constexpr (BITS == 2) {
            off[0] = half2_t{(half_t)(-(1024.f + z)), (half_t)(-(256.f + z))};
            off[1] = half2_t{(half_t)(-(64.f + z)), (half_t)(-(16.f + z))};
        } else if constexpr (BITS == 3) {
            off[0] = half2_t{(half_t)(-(1024.f + z)), (half_t)(-(128.f + z))};
        } else {
            off[0] = half2_t{(half_t)(-(1024.f + z)), (half_t)(-(1024.f + z))};
        }
    }
};

template <int BITS>
struct DequantConst<BITS, true> {
    float s, nzs;      // scale and -z * s
    __device__ __forceinline__ void set(float sc, float z)
    {
        s = sc;
        nzs = -z * sc;
    }
};

// (byte b of x) -> [b, 0x64, b, 0x64]: the byte in the low byte of both 16-bit lanes, the exponent byte of 1024.0
// above it, picked from the first source of the byte permute (selector 5 = its byte 1).  Masking the unwanted code
// bits away (with the 0x64 bytes kept by the mask) leaves the two fp16 values 1024 + c * 2^p.
__device__ __forceinline__ uint32_t spread_byte(uint32_t x, int b)
{
    return __builtin_amdgcn_perm(0x64006400u, x, 0x05000500u | ((uint32_t)b << 16) | (uint32_t)b);
}

__device__ __forceinline__ uint32_t h2_bits(half2_t v) { return __builtin_bit_cast(uint32_t, v); }

// SCALE false: the exact integers q - z are returned and the caller applies the group's scale to its sums
template <bool SCALE = true>
__device__ __forceinline__ uint32_t fp16_pair(uint32_t bits, half2_t mul, half2_t off, half2_t s2)
{
    const half2_t h = __builtin_bit_cast(half2_t, bits);
    if constexpr (SCALE) return h2_bits((h * mul + off) * s2);
    else return h2_bits(h * mul + off);
}

// 32-bit window of the unit starting at bit `bit` (compile-time after unrolling).
template <int BITS>
__device__ __forceinline__ uint32_t window(const uint32_t (&w)[BITS], int bit)
{
    const int wi = bit >> 5, sh = bit & 31;
    if (sh == 0) return w[wi];
    const uint32_t hi = wi + 1 < BITS ? w[wi + 1] : 0u;
    return __builtin_amdgcn_alignbit(hi, w[wi], (uint32_t)sh);
}

template <int BITS, bool BF16, bool SCALE = true>     // SCALE false: c was set with scale 1, the result is q - z
__device__ __forceinline__ u16x8_t dequant8(const uint32_t (&w)[BITS], int part, const DequantConst<BITS, BF16> &c)
{
    u32x4_t out;
    if constexpr (!BF16) {
        constexpr uint32_t MAGIC = 0x64006400u;   // (1024.0h, 1024.0h)
        if constexpr (BITS == 4) {
            const uint32_t x = w[part];
            const half2_t mul = {(half_t)1.f, (half_t)0.0625f};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                out[i] = fp16_pair<SCALE>(spread_byte(x, i) & (0x00F0000Fu | MAGIC), mul, c.off[0], c.s2);
        } else if constexpr (BITS == 2) {
            const uint32_t x = w[part >> 1];
            const half2_t mul0 = {(half_t)1.f, (half_t)0.25f}, mul1 = {(half_t)0.0625f, (half_t)0.015625f};
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t p = spread_byte(x, 2 * (part & 1) + i);
                out[2 * i] = fp16_pair<SCALE>(p & (0x000C0003u | MAGIC), mul0, c.off[0], c.s2);
                out[2 * i + 1] = fp16_pair<SCALE>(p & (0x00C00030u | MAGIC), mul1, c.off[1], c.s2);
            }
        } else if constexpr (BITS == 8) {
            const half2_t one = {(half_t)1.f, (half_t)1.f};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t x = w[2 * part + (i >> 1)];
                const uint32_t sel = (i & 1) ? 0x05030502u : 0x05010500u;   // [b0,0x64,b1,0x64] or [b2,0x64,b3,0x64]
                out[i] = fp16_pair<SCALE>(__builtin_amdgcn_perm(MAGIC, x, sel), one, c.off[0], c.s2);
            }
        } else {   // BITS == 3: eight codes = 24 bits starting at bit 24*part
            const uint32_t x = window<BITS>(w, 24 * part);
            const half2_t mul = {(half_t)1.f, (half_t)0.125f};
#pragma unroll
            for (int i = 0; i < 4; ++i)
                out[i] = fp16_pair<SCALE>(spread_byte(x >> (6 * i), 0) & (0x00380007u | MAGIC), mul, c.off[0], c.s2);
        }
    } else {
        constexpr uint32_t mask = (1u << BITS) - 1u;
        uint32_t x;
        int base;                                  // bit offset of code 8*part inside x
        if constexpr (BITS == 3) {
            x = window<BITS>(w, 24 * part);
            base = 0;
        } else if constexpr (BITS == 8) {
            x = 0;
            base = 0;
        } else {
            x = w[(8 * part * BITS) >> 5];
            base = (8 * part * BITS) & 31;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float f[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int e = 2 * i + h;
                uint32_t q;
                if constexpr (BITS == 8)
                    q = (w[2 * part + (e >> 2)] >> (8 * (e & 3))) & 0xffu;
                else
                    q = (x >> (base + BITS * e)) & mask;
                f[h] = (float)q * c.s + c.nzs;
            }
            typedef float float2_t __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
            out[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(float2_t{f[0], f[1]}, bf16x2_t));
        }
    }
    return __builtin_bit_cast(u16x8_t, out);
}

}  // namespace qlora
