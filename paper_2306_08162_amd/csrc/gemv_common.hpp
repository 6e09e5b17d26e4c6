// Pieces shared by the two small-token-count translation units (gemv_fwd.hip, gemv_bwd.hip).
#pragma once
#include "common.hpp"
#include "dequant.hpp"
#include "kernels.hpp"

namespace qlora {

// words per row of the bit-packed zero-points of `groups` groups (Sec. 3.2's storage count: bits per group)
inline int zero_words(int groups, int bits) { return (groups * bits + 31) / 32; }

// ---- forward: arguments of one projection, and of up to four sibling projections in one launch
struct FwdArgs {
    const uint16_t *x;
    const uint32_t *packed;
    const uint16_t *scales;
    const uint8_t *zeros;
    const uint16_t *A, *B;
    const uint16_t *t_in;     // t computed elsewhere (ranks above 32), else NULL: computed here
    uint16_t *y, *t_out;      // t_out may be NULL
    int M, N, K, r, ng;
    float sc;
    uint32_t magic;
    const uint32_t *zpacked;  // zero-points in their bit-packed storage form [N, zw] (then `zeros` is not read), or NULL
    int zw;                   // words per row of zpacked
};

// Sibling projections (q/k/v, gate/up) read the same x: one launch serves up to four of them.  They share M, K, the
// code width, the grouping and the rank; workgroups [wg_end[i-1], wg_end[i]) belong to projection i.
struct FwdMulti {
    FwdArgs p[MAX_SIBLINGS];
    int wg_end[MAX_SIBLINGS];
    int count;
};

// the forward kernels of one code width (each width is its own translation unit).  false: nothing was launched
// (bit-packed zero-points were handed in and no kernel that reads them takes the shape)
template <int BITS>
bool launch_fwd_small_bits(const FwdMulti &m, int rg, bool bf16, hipStream_t s);

// zero-point of group g from a row of bit-packed zero-points (little-endian stream of BITS-wide fields)
template <int BITS>
__device__ __forceinline__ uint32_t packed_zero(const uint32_t *row_words, int g)
{
    const int o = g * BITS, w = o >> 5, sh = o & 31;
    uint32_t v = row_words[w] >> sh;
    if (BITS == 3 && sh > 29) v |= row_words[w + 1] << (32 - sh);
    return v & ((1u << BITS) - 1u);
}

namespace {


template <bool BF16>
__device__ __forceinline__ float4_t mfma16(u16x8_t a, u16x8_t b, float4_t c)
{
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                       c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c,
                                                      0, 0, 0);
}

template <int BITS>
__device__ __forceinline__ void load_words(const uint32_t *__restrict__ p, uint32_t (&w)[BITS])
{
    if constexpr (BITS == 2) {
        const u32x2_t v = *(const u32x2_t *)p;
        w[0] = v[0];
        w[1] = v[1];
    } else if constexpr (BITS == 4) {
        const u32x4_t v = *(const u32x4_t *)p;
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = v[i];
    } else if constexpr (BITS == 8) {
        const u32x4_t v0 = *(const u32x4_t *)p, v1 = *(const u32x4_t *)(p + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            w[i] = v0[i];
            w[4 + i] = v1[i];
        }
    } else {
#pragma unroll
        for (int i = 0; i < BITS; ++i) w[i] = p[i];
    }
}

__device__ __forceinline__ int group_of(int k, uint32_t magic) { return magic ? (int)__umulhi((uint32_t)(k >> 5), magic) : (k >> 5); }

constexpr u16x8_t ZERO8 = {0, 0, 0, 0, 0, 0, 0, 0};

inline uint32_t group_magic(int G)
{
    const uint32_t d = (uint32_t)(G / 32);
    return d == 1 ? 0u : (uint32_t)(0x100000000ull / d) + 1u;
}

#define QLORA_BITS_DTYPE(FN, ...)                              \
    do {                                                       \
        if (p.bf16) {                                          \
            switch (p.bits) {                                  \
            case 2: FN<2, true>(__VA_ARGS__); break;           \
            case 3: FN<3, true>(__VA_ARGS__); break;           \
            case 4: FN<4, true>(__VA_ARGS__); break;           \
            default: FN<8, true>(__VA_ARGS__); break;          \
            }                                                  \
        } else {                                               \
            switch (p.bits) {                                  \
            case 2: FN<2, false>(__VA_ARGS__); break;          \
            case 3: FN<3, false>(__VA_ARGS__); break;          \
            case 4: FN<4, false>(__VA_ARGS__); break;          \
            default: FN<8, false>(__VA_ARGS__); break;         \
            }                                                  \
        }                                                      \
    } while (0)

}  // namespace

}  // namespace qlora
