// Shared device helpers of the HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qlora {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8_t __attribute__((ext_vector_type(8)));

constexpr int WAVE = 64;

// ---- 16-bit float <-> fp32 on raw bit patterns -----------------------------

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                              // round to nearest even
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t b)
{
    union { uint16_t u; half_t h; } c;
    c.u = b;
    return (float)c.h;
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float f)
{
    union { uint16_t u; half_t h; } c;
    c.h = (half_t)f;  // v_cvt_f16_f32: round to nearest even
    return c.u;
}

template <bool BF16>
__device__ __forceinline__ float ld16(const uint16_t *p)
{
    return BF16 ? bf16_bits_to_f32(*p) : f16_bits_to_f32(*p);
}

template <bool BF16>
__device__ __forceinline__ float cvt16(uint16_t b)
{
    return BF16 ? bf16_bits_to_f32(b) : f16_bits_to_f32(b);
}

template <bool BF16>
__device__ __forceinline__ uint16_t to16(float f)
{
    return BF16 ? f32_to_bf16_bits(f) : f32_to_f16_bits(f);
}

// ---- packed codes -----------------------------------------------------------

// Code k of one packed row: little-endian bit stream, code k at stream bits [BITS*k, BITS*k+BITS).
template <int BITS>
__device__ __forceinline__ uint32_t code_at(const uint32_t *__restrict__ row, int k)
{
    constexpr uint32_t mask = (1u << BITS) - 1u;
    if constexpr (BITS == 3) {
        const int o = 3 * k, w = o >> 5, sh = o & 31;
        uint32_t q = row[w] >> sh;
        if (sh > 29) q |= row[w + 1] << (32 - sh);
        return q & mask;
    } else {
        constexpr int per = 32 / BITS;
        return (row[k / per] >> (BITS * (k % per))) & mask;
    }
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

// Direct-to-LDS load: every lane fetches 16 bytes from base + its own 32-bit byte offset, and the 64 pieces land
// contiguously at the wave-uniform LDS byte address `lds` (1 KB, lane l at lds + 16 l).  Written as assembly so that
// the compiler does not order it against the LDS reads around it; completion is tracked by the vector-memory
// counter, which the caller waits on itself (the compiler does not see these loads).
__device__ __forceinline__ void dma16(const void *base, uint32_t byte_offset, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 ::"v"(byte_offset), "s"(base), "s"(lds)
                 : "memory");   // m0 is reserved by the compiler: it never keeps a value there across other code
}

// The 4-byte form: lane l's dword lands at lds + 4 l (256 bytes per instruction).
__device__ __forceinline__ void dma4(const void *base, uint32_t byte_offset, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 ::"v"(byte_offset), "s"(base), "s"(lds)
                 : "memory");
}

// The 16-byte form with a full address per lane (the lanes of one request may read different arrays).
__device__ __forceinline__ void dma16_at(const void *lane_address, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 ::"v"(lane_address), "s"(lds)
                 : "memory");
}

}  // namespace qlora
