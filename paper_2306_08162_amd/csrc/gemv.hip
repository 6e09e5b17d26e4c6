// Small token counts (M <= 64): the pass is bound by streaming the packed weight once from HBM, so every lane
// fetches its own MFMA fragment of packed words straight from global memory, dequantises it in registers and
// feeds v_mfma_f32_16x16x32; nothing but partial sums goes through LDS.  (Limitations of the paper: the compressed
// weight cuts the memory traffic of both passes; this is the regime where that shows.)
//
//   forward   y [M,N] = x  Wd^T + sc * t B^T     one workgroup per 16 weight rows, its 4 waves split K
//   backward  dX[M,K] = dY Wd   + sc * u A       one workgroup per 128 weight columns and slice of rows;
//             the contraction runs over rows n, so a lane gathers one word from each of 8 rows and transposes
//             the 8 x 8 block of codes in registers (Sec. 3.1: transpose + unpack + matmul in one kernel)
#include "common.hpp"
#include "dequant.hpp"
#include "kernels.hpp"

namespace qlora {

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

// ------------------------------------------------------------------------------------------------- forward
constexpr int FW_U = 4;   // iterations (128 codes per row each) whose loads are in flight together

template <int BITS, bool BF16, int MB>
__global__ __launch_bounds__(256) void gemv_fwd_kernel(const uint16_t *__restrict__ x, const uint32_t *__restrict__ packed,
                                                       const uint16_t *__restrict__ scales, const uint8_t *__restrict__ zeros,
                                                       const uint16_t *__restrict__ t, const uint16_t *__restrict__ B,
                                                       uint16_t *__restrict__ y, int M, int N, int K, int r, float sc,
                                                       uint32_t magic, int ng)
{
    __shared__ float red[4][MB][16][17];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.x * 16, n = min(n0 + li, N - 1);
    const int Kw = K * BITS / 32;
    const uint32_t *wrow = packed + (long)n * Kw;
    const uint16_t *xrow[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) xrow[mb] = x + (long)min(mb * 16 + li, M - 1) * K;

    float4_t acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb] = float4_t{0.f, 0.f, 0.f, 0.f};

    const int iters = (K + 127) / 128;          // wave w takes iterations w, w+4, ...: neighbours read neighbouring bytes
    for (int it0 = wave; it0 < iters; it0 += 4 * FW_U) {
        uint32_t w[FW_U][BITS];
        uint16_t sraw[FW_U];
        uint8_t zraw[FW_U];
        bool ok[FW_U];
        u16x8_t xf[FW_U][MB][4];
#pragma unroll
        for (int u = 0; u < FW_U; ++u) {
            const int kb = (it0 + 4 * u) * 128 + 32 * q;
            ok[u] = kb < K;
            const int kc = ok[u] ? kb : 0;
            load_words<BITS>(wrow + (kc >> 5) * BITS, w[u]);
            const long gi = (long)n * ng + group_of(kc, magic);
            sraw[u] = scales[gi];
            zraw[u] = zeros[gi];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int s = 0; s < 4; ++s) xf[u][mb][s] = *(const u16x8_t *)(xrow[mb] + kc + 8 * s);
        }
#pragma unroll
        for (int u = 0; u < FW_U; ++u) {
            DequantConst<BITS, BF16> dq;
            dq.set(ok[u] ? f16_bits_to_f32(sraw[u]) : 0.f, (float)zraw[u]);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const u16x8_t wf = dequant8<BITS, BF16>(w[u], s, dq);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) acc[mb] = mfma16<BF16>(xf[u][mb][s], wf, acc[mb]);   // D[m = 4q+v][n = li]
            }
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][mb][4 * q + v][li] = acc[mb][v];
    __syncthreads();
    for (int e = threadIdx.x; e < MB * 256; e += 256) {
        const int mb = e >> 8, ml = (e >> 4) & 15, nl = e & 15;
        const int m = mb * 16 + ml, nn = n0 + nl;
        if (m >= M || nn >= N) continue;
        float v = ((red[0][mb][ml][nl] + red[1][mb][ml][nl]) + red[2][mb][ml][nl]) + red[3][mb][ml][nl];
        float lo = 0.f;
        for (int j = 0; j < r; ++j) lo += cvt16<BF16>(t[(long)m * r + j]) * cvt16<BF16>(B[(long)nn * r + j]);
        y[(long)m * N + nn] = to16<BF16>(v + sc * lo);
    }
}

// ------------------------------------------------------------------------------------------------ backward
// Workgroup (cb, sp): weight columns [128 cb, +128), rows n of slice sp; wave w takes 32-row chunks w, w+4, ...
// Lane (wc = lane % 16, q = lane / 16) loads the word holding columns 128 cb + 8 wc .. + 8 from rows
// chunk*32 + 8 q + e, e = 0..7.  MFMA number c of a chunk multiplies dY[m, 32 rows] with the codes at column
// 8 wc + c of those rows: D_c[m][k = 128 cb + 8 wc + c].
constexpr int BW_COLS = 128;

// Column c (compile-time) of an 8-row block of words holding 8 codes each, as eight 16-bit floats
// s_e * (q_e - z_e), rows e = 0..7.  Only widths whose 8 codes fill a whole number of bytes go through here.
template <int BITS, bool BF16>
__device__ __forceinline__ u16x8_t column8(const uint32_t (&w)[8], int c, const float (&s)[8], const float (&z)[8])
{
    u16x8_t out;
    constexpr uint32_t mask = (1u << BITS) - 1u;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = ((float)((w[e] >> (BITS * c)) & mask) - z[e]) * s[e];
        out[e] = to16<BF16>(v);
    }
    return out;
}

template <int BITS, bool BF16, int MB>
__global__ __launch_bounds__(256) void gemv_bwd_kernel(const uint16_t *__restrict__ dy, const uint32_t *__restrict__ packed,
                                                       const uint16_t *__restrict__ scales, const uint8_t *__restrict__ zeros,
                                                       float *__restrict__ partial, int M, int N, int K, uint32_t magic,
                                                       int ng, int rows_per_slice)
{
    // 8 codes of a row = BITS bytes; a lane's "word" is the 32-bit window starting at that byte
    __shared__ float red[4][16][BW_COLS + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wc = lane & 15, q = lane >> 4;
    const int kcol = blockIdx.x * BW_COLS + 8 * wc;          // first of this lane's 8 columns
    const bool kok = kcol < K;
    const int kc = kok ? kcol : 0;
    const int Kw = K * BITS / 32;
    const int g = group_of(kc, magic);
    const int nbeg = blockIdx.y * rows_per_slice, nend = min(N, nbeg + rows_per_slice);
    const uint8_t *pbytes = (const uint8_t *)packed;

    float4_t acc[MB][8];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[mb][c] = float4_t{0.f, 0.f, 0.f, 0.f};

    for (int n0 = nbeg + wave * 32; n0 < nend; n0 += 128) {
        uint32_t w[8];
        float s[8], z[8];
        u16x8_t df[MB];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int n = n0 + 8 * q + e;
            const bool ok = kok && n < nend;
            const int nc = min(n, N - 1);
            const uint8_t *src = pbytes + (long)nc * Kw * 4 + (long)(kc >> 3) * BITS;   // byte address of 8 codes
            if constexpr (BITS == 4) {
                w[e] = *(const uint32_t *)src;
            } else if constexpr (BITS == 8) {
                w[e] = 0;   // handled below with two words
            } else if constexpr (BITS == 2) {
                w[e] = *(const uint16_t *)src;
            } else {        // 3 bits: 3 bytes, not word aligned
                uint32_t v = 0;
#pragma unroll
                for (int b = 0; b < BITS; ++b) v |= (uint32_t)src[b] << (8 * b);
                w[e] = v;
            }
            const long gi = (long)nc * ng + g;
            s[e] = ok ? f16_bits_to_f32(scales[gi]) : 0.f;
            z[e] = (float)zeros[gi];
        }
        uint32_t w2[8];     // second word for 8-bit codes (columns 4..7)
        if constexpr (BITS == 8) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int nc = min(n0 + 8 * q + e, N - 1);
                const u32x2_t v = *(const u32x2_t *)(pbytes + (long)nc * Kw * 4 + (long)(kc >> 3) * 8);
                w[e] = v[0];
                w2[e] = v[1];
            }
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int m = min(mb * 16 + wc, M - 1);
            const int nn = n0 + 8 * q;                       // 8 consecutive rows n = contraction indices of this lane
            const bool in = nn < nend;                       // N % 8 == 0 and slices are multiples of 32: all or nothing
            df[mb] = *(const u16x8_t *)(dy + (long)m * N + (in ? nn : 0));
            if (!in) df[mb] = u16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            u16x8_t wf;
            if constexpr (BITS == 8)
                wf = c < 4 ? column8<8, BF16>(w, c, s, z) : column8<8, BF16>(w2, c - 4, s, z);
            else
                wf = column8<BITS, BF16>(w, c, s, z);
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[mb][c] = mfma16<BF16>(df[mb], wf, acc[mb][c]);   // D[m = 4q+v][col wc]
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        if (mb) __syncthreads();
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][4 * q + v][8 * wc + c] = acc[mb][c][v];
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * BW_COLS; e += 256) {
            const int ml = e / BW_COLS, kl = e % BW_COLS;
            const int m = mb * 16 + ml, k = blockIdx.x * BW_COLS + kl;
            if (m >= M || k >= K) continue;
            const float v = ((red[0][ml][kl] + red[1][ml][kl]) + red[2][ml][kl]) + red[3][ml][kl];
            partial[((long)blockIdx.y * M + m) * K + k] = v;
        }
    }
}

// dx[m,k] = sum over slices (in order) of partial + sc * sum_j u[m,j] A[j,k]
template <bool BF16>
__global__ __launch_bounds__(256) void gemv_bwd_finish_kernel(const float *__restrict__ partial, const uint16_t *__restrict__ u,
                                                              const uint16_t *__restrict__ A, uint16_t *__restrict__ dx,
                                                              int M, int K, int r, float sc, int slices)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)M * K) return;
    const int m = (int)(idx / K), k = (int)(idx % K);
    float v = 0.f;
    for (int s = 0; s < slices; ++s) v += partial[(long)s * M * K + idx];
    float lo = 0.f;
    for (int j = 0; j < r; ++j) lo += cvt16<BF16>(u[(long)m * r + j]) * cvt16<BF16>(A[(long)j * K + k]);
    dx[idx] = to16<BF16>(v + sc * lo);
}

template <int BITS, bool BF16>
void launch_fwd_mb(const Problem &p, const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                   const void *t, const void *B, void *y, uint32_t magic, hipStream_t s)
{
    const dim3 grid((p.N + 15) / 16), block(256);
    const int ng = p.K / p.G;
#define QLORA_FWD(MBV)                                                                                              \
    hipLaunchKernelGGL((gemv_fwd_kernel<BITS, BF16, MBV>), grid, block, 0, s, (const uint16_t *)x, packed,           \
                       (const uint16_t *)scales, zeros, (const uint16_t *)t, (const uint16_t *)B, (uint16_t *)y, p.M, \
                       p.N, p.K, p.r, p.sc, magic, ng)
    switch ((p.M + 15) / 16) {
    case 1: QLORA_FWD(1); break;
    case 2: QLORA_FWD(2); break;
    case 3: QLORA_FWD(3); break;
    default: QLORA_FWD(4); break;
    }
#undef QLORA_FWD
}

template <int BITS, bool BF16>
void launch_bwd_mb(const Problem &p, const void *dy, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                   const void *u, const void *A, void *dx, float *partial, uint32_t magic, hipStream_t s)
{
    const int slices = gemv_bwd_slices(p.N, p.K);
    const int rows_per_slice = ((p.N + slices - 1) / slices + 31) / 32 * 32;
    const dim3 grid((p.K + BW_COLS - 1) / BW_COLS, slices), block(256);
    const int ng = p.K / p.G;
#define QLORA_BWD(MBV)                                                                                         \
    hipLaunchKernelGGL((gemv_bwd_kernel<BITS, BF16, MBV>), grid, block, 0, s, (const uint16_t *)dy, packed,     \
                       (const uint16_t *)scales, zeros, partial, p.M, p.N, p.K, magic, ng, rows_per_slice)
    switch ((p.M + 15) / 16) {
    case 1: QLORA_BWD(1); break;
    case 2: QLORA_BWD(2); break;
    case 3: QLORA_BWD(3); break;
    default: QLORA_BWD(4); break;
    }
#undef QLORA_BWD
    const long n = (long)p.M * p.K;
    hipLaunchKernelGGL((gemv_bwd_finish_kernel<BF16>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, partial,
                       (const uint16_t *)u, (const uint16_t *)A, (uint16_t *)dx, p.M, p.K, p.r, p.sc, slices);
}

inline uint32_t group_magic(int G)
{
    const uint32_t d = (uint32_t)(G / 32);
    return d == 1 ? 0u : (uint32_t)(0x100000000ull / d) + 1u;
}

}  // namespace

int gemv_bwd_slices(int N, int K)
{
    const int colblocks = (K + BW_COLS - 1) / BW_COLS;
    int slices = (512 + colblocks - 1) / colblocks;      // aim at >= 512 workgroups
    const int max_slices = (N + 127) / 128;              // at least one 32-row chunk per wave
    if (slices > max_slices) slices = max_slices;
    return slices < 1 ? 1 : slices;
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

void launch_fwd_small(const Problem &p, const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                      const void *t, const void *B, void *y, hipStream_t s)
{
    const uint32_t magic = group_magic(p.G);
    QLORA_BITS_DTYPE(launch_fwd_mb, p, x, packed, scales, zeros, t, B, y, magic, s);
}

void launch_bwd_dx_small(const Problem &p, const void *dy, const uint32_t *packed, const void *scales,
                         const uint8_t *zeros, const void *u, const void *A, void *dx, float *partial, hipStream_t s)
{
    const uint32_t magic = group_magic(p.G);
    QLORA_BITS_DTYPE(launch_bwd_mb, p, dy, packed, scales, zeros, u, A, dx, partial, magic, s);
}

}  // namespace qlora
