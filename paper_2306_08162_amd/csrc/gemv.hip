// Small token counts: the pass is bound by streaming the packed weight once from HBM (Limitations of the paper:
// the compressed weight cuts the memory traffic of both passes; this is the regime where that shows).  Every lane
// fetches its own MFMA fragment of packed words straight from global memory, dequantises it in registers and feeds
// v_mfma_f32_16x16x32; partial sums go through LDS (and, up to 32 token rows, so do x and A: see the staged
// forward kernel).  Launches are what the pass is made of at this size, so the rank-r products ride along: one
// launch forward, two backward.
//
//   forward  (M <= 64)  y = x Wd^T + sc * t B^T with t = x A^T computed by the same MFMAs (one extra fragment of
//            A per k-step); one workgroup per 16 weight rows (up to four such blocks), its waves split K.
//   backward (M <= 16)  kernel 1: partial dX = dY Wd over row slices of the weight, and partial u = dY B.  The
//            contraction runs over the weight's rows n, so a lane gathers the same few words from 8 consecutive
//            rows and transposes the 8 x CL block of codes in registers (Sec. 3.1: transpose + unpack + matmul in one
//            kernel).  kernel 2: sums the slices, adds sc * u A, and forms dA = sc u^T x and dB = sc dY^T t.
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

constexpr u16x8_t ZERO8 = {0, 0, 0, 0, 0, 0, 0, 0};

// ------------------------------------------------------------------------------------------------- forward
#ifndef QLORA_FW_U
#define QLORA_FW_U 4
#endif
constexpr int FW_U = QLORA_FW_U;   // iterations (128 codes per row each) whose loads are in flight together

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
};

// Sibling projections (q/k/v, gate/up) read the same x: one launch serves up to four of them.  They share M, K, the
// code width, the grouping and the rank; workgroups [wg_end[i-1], wg_end[i]) belong to projection i.
struct FwdMulti {
    FwdArgs p[MAX_SIBLINGS];
    int wg_end[MAX_SIBLINGS];
    int count;
};

template <int BITS, bool BF16, int MB, int RG, int NW, int NB>   // RG: 16-column groups of t formed here (0: none);
                                                                  // NW waves; NB 16-row weight blocks per workgroup
__global__ __launch_bounds__(NW * 64) void gemv_fwd_kernel(const FwdArgs a)
{
    constexpr int RGS = RG > 0 ? RG : 1, NT = NW * 64;
    __shared__ float red[NW][MB][NB][16][17];
    __shared__ float tred[NW][MB][RGS][16][17];
    constexpr int TC = RG > 0 ? RG * 16 : 64;      // columns of t kept in LDS
    __shared__ float tfull[MB * 16][TC + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.x * 16 * NB;
    const int K = a.K, Kw = K * BITS / 32, r = a.r;
    // the activation (and A) fragments of a k-step are fetched once and used for all NB weight blocks: they, not the
    // packed weight, are most of what a workgroup pulls through its L1
    int nrow[NB];
    const uint32_t *wrow[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        nrow[nb] = min(n0 + nb * 16 + li, a.N - 1);
        wrow[nb] = a.packed + (long)nrow[nb] * Kw;
    }
    const uint16_t *xrow[MB], *arow[RGS];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) xrow[mb] = a.x + (long)min(mb * 16 + li, a.M - 1) * K;
    bool aval[RGS];
#pragma unroll
    for (int g = 0; g < RGS; ++g) {
        aval[g] = RG > 0 && g * 16 + li < r;
        arow[g] = a.A + (long)(RG > 0 ? min(g * 16 + li, r - 1) : 0) * K;
    }

    float4_t acc[MB][NB], tacc[MB][RGS];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int g = 0; g < RGS; ++g) tacc[mb][g] = float4_t{0.f, 0.f, 0.f, 0.f};
    }

    const int iters = (K + 127) / 128;          // wave w takes iterations w, w+NW, ...: neighbours read neighbouring bytes
    for (int it0 = wave; it0 < iters; it0 += NW * FW_U) {
        uint32_t w[FW_U][NB][BITS];
        uint16_t sraw[FW_U][NB];
        uint8_t zraw[FW_U][NB];
        bool ok[FW_U];
        u16x8_t xf[FW_U][MB][4], af[FW_U][RGS][4];
#pragma unroll
        for (int u = 0; u < FW_U; ++u) {
            const int kb = (it0 + NW * u) * 128 + 32 * q;
            ok[u] = kb < K;
            const int kc = ok[u] ? kb : 0;
            const int grp = group_of(kc, a.magic);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                load_words<BITS>(wrow[nb] + (kc >> 5) * BITS, w[u][nb]);
                const long gi = (long)nrow[nb] * a.ng + grp;
                sraw[u][nb] = a.scales[gi];
                zraw[u][nb] = a.zeros[gi];
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) xf[u][mb][s] = *(const u16x8_t *)(xrow[mb] + kc + 8 * s);
                if constexpr (RG > 0) {
#pragma unroll
                    for (int g = 0; g < RG; ++g)
                        af[u][g][s] = aval[g] ? *(const u16x8_t *)(arow[g] + kc + 8 * s) : ZERO8;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < FW_U; ++u) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                DequantConst<BITS, BF16> dq;
                dq.set(ok[u] ? f16_bits_to_f32(sraw[u][nb]) : 0.f, (float)zraw[u][nb]);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const u16x8_t wf = dequant8<BITS, BF16>(w[u][nb], s, dq);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        acc[mb][nb] = mfma16<BF16>(xf[u][mb][s], wf, acc[mb][nb]);    // D[m = 4q+v][n = li]
                }
            }
            if constexpr (RG > 0) {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int g = 0; g < RG; ++g) {
                        const u16x8_t afz = ok[u] ? af[u][g][s] : ZERO8;
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) tacc[mb][g] = mfma16<BF16>(xf[u][mb][s], afz, tacc[mb][g]);   // D[m][j = li]
                    }
            }
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) red[wave][mb][nb][4 * q + v][li] = acc[mb][nb][v];
            if constexpr (RG > 0) {
#pragma unroll
                for (int g = 0; g < RG; ++g) tred[wave][mb][g][4 * q + v][li] = tacc[mb][g][v];
            }
        }
    __syncthreads();
    // t for all token rows of the call (every workgroup computes the same t; workgroup 0 hands it out)
    if constexpr (RG > 0) {
        for (int e = threadIdx.x; e < MB * 16 * RG * 16; e += NT) {
            const int m = e / (RG * 16), j = e % (RG * 16);
            float tv = 0.f;
            if (j < r && m < a.M) {
                const int mb = m >> 4, ml = m & 15, g = j >> 4, jl = j & 15;
#pragma unroll
                for (int w = 0; w < NW; ++w) tv += tred[w][mb][g][ml][jl];
                tv = cvt16<BF16>(to16<BF16>(tv));          // the value every consumer of t sees
                if (blockIdx.x == 0 && a.t_out) a.t_out[(long)m * r + j] = to16<BF16>(tv);
            }
            tfull[m][j] = tv;
        }
    } else {
        for (int e = threadIdx.x; e < a.M * r; e += NT) tfull[e / r][e % r] = cvt16<BF16>(a.t_in[e]);
    }
    __syncthreads();
    for (int e = threadIdx.x; e < MB * NB * 256; e += NT) {
        const int mb = e / (NB * 256), nb = (e >> 8) % NB, ml = (e >> 4) & 15, nl = e & 15;
        const int m = mb * 16 + ml, nn = n0 + nb * 16 + nl;
        if (m >= a.M || nn >= a.N) continue;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) v += red[w][mb][nb][ml][nl];
        float lo = 0.f;
        for (int j0 = 0; j0 < r; j0 += 8) {
            const u16x8_t bv = *(const u16x8_t *)(a.B + (long)nn * r + j0);
#pragma unroll
            for (int h = 0; h < 8; ++h) lo += tfull[m][j0 + h] * cvt16<BF16>(bv[h]);
        }
        a.y[(long)m * a.N + nn] = to16<BF16>(v + a.sc * lo);
    }
}

// ------------------------------------------------------------------------------- forward, staged activations
// Same products as gemv_fwd_kernel for up to two 16-row token blocks, with a different route for x and A.  A lane's
// MFMA fragment of x is 16 bytes out of each of 16 different rows: fetched as such, a wave touches 64 separate
// 64-byte pieces per instruction and the pass is bound by that, not by the packed weight.  Here every wave copies
// its 128-column slice of x and A straight into LDS with row-contiguous requests (global_load_lds, 16 lanes per
// 256-byte row segment, no registers in between) and takes the fragments from there.  The slices are private to
// the wave, two deep, so the loop has no workgroup barrier; the packed words still go from global memory to
// registers, a batch of iterations ahead.
//
// LDS slice of one 16-row block: 16 rows x 16 pieces of 16 bytes; piece c of row w sits in slot 16 w + (c ^ w), so
// the fragment reads of 16 rows at one piece index fall on 16 different bank groups.
constexpr int ST_BLOCK = 4096;      // bytes of one 16-row x 128-column block
#ifndef QLORA_ST_U
#define QLORA_ST_U 4
#endif
constexpr int ST_U = QLORA_ST_U;    // iterations whose packed words are requested together

__device__ __forceinline__ void dma16(const void *base, uint32_t byte_offset, uint32_t lds)
{
    // lane l of the wave writes its 16 bytes to LDS byte address lds + 16 l; completion counts on vmcnt
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(byte_offset), "s"(base), "s"(lds)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ void wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

template <int BITS, bool BF16, int MB, int RG, int NW, int NB>   // NB: 16-row weight blocks per workgroup
__device__ __forceinline__ void gemv_fwd_staged_body(const FwdArgs &a, const int wg)   // wg: workgroup index inside the projection
{
    constexpr int RGS = RG > 0 ? RG : 1, NT = NW * 64;
    constexpr int BLOCKS = MB + RG;                 // 16-row blocks per slice: x blocks, then A blocks
    constexpr int ND = 4 * BLOCKS;                  // LDS-DMA instructions per slice
    extern __shared__ __attribute__((aligned(16))) uint8_t stage[];   // [NW][2][BLOCKS][ST_BLOCK]
    // a wave's partial sums go where its slices were, once it has used the last of them
    constexpr int WAVE_STAGE = 2 * BLOCKS * ST_BLOCK;
    static_assert((MB * NB + MB * RGS) * 16 * 17 * 4 <= WAVE_STAGE, "partial sums fit in the wave's slices");
    auto red = [&](int w, int mb, int nb, int row, int col) -> float & {
        return ((float *)(stage + (size_t)w * WAVE_STAGE))[((mb * NB + nb) * 16 + row) * 17 + col];
    };
    auto tred = [&](int w, int mb, int g, int row, int col) -> float & {
        return ((float *)(stage + (size_t)w * WAVE_STAGE))[((MB * NB + mb * RGS + g) * 16 + row) * 17 + col];
    };
    constexpr int TC = RG > 0 ? RG * 16 : 64;
    __shared__ float tfull[MB * 16][TC + 1];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, q = lane >> 4;
    const int n0 = wg * 16 * NB;
    const int K = a.K, Kw = K * BITS / 32, r = a.r;
    int nrow[NB];
    const uint32_t *wrow[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        nrow[nb] = min(n0 + nb * 16 + li, a.N - 1);
        wrow[nb] = a.packed + (long)nrow[nb] * Kw;
    }
    // this lane's part of a slice copy: instruction j of a block moves rows 4j + lane/16; the lane fetches the
    // piece that belongs in its slot
    uint32_t src_off[BLOCKS][4];                    // byte offset of (row, piece) at column 0 of the slice
#pragma unroll
    for (int b = 0; b < BLOCKS; ++b)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int w16 = 4 * j + (lane >> 4), piece = (lane & 15) ^ w16;
            const int row = b < MB ? min(b * 16 + w16, a.M - 1) : min((b - MB) * 16 + w16, r - 1);   // clamped rows
            src_off[b][j] = (uint32_t)(((long)row * K + 8 * piece) * 2);                             // repeat a valid one
        }
    const uint32_t my_stage = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)stage +
                              (uint32_t)wave * WAVE_STAGE;
    const int iters = (K + 127) / 128;
    const int n_it = wave < iters ? (iters - wave + NW - 1) / NW : 0;      // this wave's iterations: wave, wave+NW, ..
    auto issue_slice = [&](int i, int buf) {
        const int k0 = (wave + NW * i) * 128;
#pragma unroll
        for (int b = 0; b < BLOCKS; ++b)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // pieces past K (last iteration of a K that is not a multiple of 128) re-read column 0: their
                // weights are scaled by zero and their A fragments replaced by zero below
                const int piece = (lane & 15) ^ (4 * j + (lane >> 4));
                const uint32_t kb = k0 + 8 * piece < K ? (uint32_t)k0 * 2u : (uint32_t)(-(8 * piece)) * 2u;
                dma16(b < MB ? (const void *)a.x : (const void *)a.A, src_off[b][j] + kb,
                      my_stage + (uint32_t)((buf * BLOCKS + b) * ST_BLOCK + j * 1024));
            }
    };

    // the rows of B this thread's outputs need at the very end: requested now, so they are not one more round trip then
    constexpr int EPT = (MB * NB * 256 + NT - 1) / NT;
    u16x8_t bpre[EPT][2 * RGS];
    if constexpr (RG > 0) {
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int e = threadIdx.x + x * NT, nn = n0 + ((e >> 8) % NB) * 16 + (e & 15);
            const bool live = e < MB * NB * 256 && nn < a.N;
#pragma unroll
            for (int h = 0; h < 2 * RG; ++h)
                bpre[x][h] = (live && 8 * h < r) ? *(const u16x8_t *)(a.B + (long)nn * r + 8 * h) : ZERO8;
        }
    }

    float4_t acc[MB][NB], tacc[MB][RGS];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int g = 0; g < RGS; ++g) tacc[mb][g] = float4_t{0.f, 0.f, 0.f, 0.f};
    }

    for (int i0 = 0; i0 < n_it; i0 += ST_U) {
        uint32_t w[ST_U][NB][BITS];
        uint16_t sraw[ST_U][NB];
        uint8_t zraw[ST_U][NB];
        bool ok[ST_U];
#pragma unroll
        for (int u = 0; u < ST_U; ++u) {
            const int kb = (wave + NW * (i0 + u)) * 128 + 32 * q;
            ok[u] = kb < K;                           // also false for iterations past the wave's last
            const int kc = ok[u] ? kb : 0;
            const int grp = group_of(kc, a.magic);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                load_words<BITS>(wrow[nb] + (kc >> 5) * BITS, w[u][nb]);
                const long gi = (long)nrow[nb] * a.ng + grp;
                sraw[u][nb] = a.scales[gi];
                zraw[u][nb] = a.zeros[gi];
            }
        }
        if (i0 == 0) {      // the first two slices go out behind the first batch of packed words, not ahead of it
            issue_slice(0, 0);
            if (n_it > 1) issue_slice(1, 1);
        }
#pragma unroll
        for (int u = 0; u < ST_U; ++u) {
            const int i = i0 + u;
            if (i >= n_it) break;
            // slice i has landed when at most the ND copies of slice i+1 (issued after it) are still in flight
            if (i + 1 < n_it) wait_vm<ND>(); else wait_vm<0>();
            const uint8_t *buf = stage + (size_t)wave * WAVE_STAGE + (size_t)(u & 1) * (BLOCKS * ST_BLOCK);
            u16x8_t xf[MB][4], af[RGS][4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int slot = li * 16 + ((4 * q + s) ^ li);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) xf[mb][s] = *(const u16x8_t *)(buf + mb * ST_BLOCK + slot * 16);
                if constexpr (RG > 0) {
#pragma unroll
                    for (int g = 0; g < RG; ++g) {
                        const u16x8_t v = *(const u16x8_t *)(buf + (MB + g) * ST_BLOCK + slot * 16);
                        af[g][s] = (ok[u] && g * 16 + li < r) ? v : ZERO8;
                    }
                }
            }
            wait_lds();                               // the fragments are in registers: the slice may be overwritten
            if (i + 2 < n_it) issue_slice(i + 2, u & 1);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                DequantConst<BITS, BF16> dq;
                dq.set(ok[u] ? f16_bits_to_f32(sraw[u][nb]) : 0.f, (float)zraw[u][nb]);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const u16x8_t wf = dequant8<BITS, BF16>(w[u][nb], s, dq);
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb)
                        acc[mb][nb] = mfma16<BF16>(xf[mb][s], wf, acc[mb][nb]);       // D[m = 4q+v][n = li]
                }
            }
            if constexpr (RG > 0) {
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int g = 0; g < RG; ++g)
#pragma unroll
                        for (int mb = 0; mb < MB; ++mb) tacc[mb][g] = mfma16<BF16>(xf[mb][s], af[g][s], tacc[mb][g]);
            }
        }
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) red(wave, mb, nb, 4 * q + v, li) = acc[mb][nb][v];
            if constexpr (RG > 0) {
#pragma unroll
                for (int g = 0; g < RG; ++g) tred(wave, mb, g, 4 * q + v, li) = tacc[mb][g][v];
            }
        }
    __syncthreads();
    if constexpr (RG > 0) {
        for (int e = threadIdx.x; e < MB * 16 * RG * 16; e += NT) {
            const int m = e / (RG * 16), j = e % (RG * 16);
            float tv = 0.f;
            if (j < r && m < a.M) {
                const int mb = m >> 4, ml = m & 15, g = j >> 4, jl = j & 15;
#pragma unroll
                for (int w = 0; w < NW; ++w) tv += tred(w, mb, g, ml, jl);
                tv = cvt16<BF16>(to16<BF16>(tv));          // the value every consumer of t sees
                if (wg == 0 && a.t_out) a.t_out[(long)m * r + j] = to16<BF16>(tv);
            }
            tfull[m][j] = tv;
        }
    } else {
        for (int e = threadIdx.x; e < a.M * r; e += NT) tfull[e / r][e % r] = cvt16<BF16>(a.t_in[e]);
    }
    __syncthreads();
#pragma unroll
    for (int x = 0; x < EPT; ++x) {
        const int e = threadIdx.x + x * NT;
        const int mb = e / (NB * 256), nb = (e >> 8) % NB, ml = (e >> 4) & 15, nl = e & 15;
        const int m = mb * 16 + ml, nn = n0 + nb * 16 + nl;
        if (e >= MB * NB * 256 || m >= a.M || nn >= a.N) continue;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) v += red(w, mb, nb, ml, nl);
        float lo = 0.f;
        if constexpr (RG > 0) {
#pragma unroll
            for (int h = 0; h < 2 * RG; ++h)
#pragma unroll
                for (int c = 0; c < 8; ++c) lo += tfull[m][8 * h + c] * cvt16<BF16>(bpre[x][h][c]);   // zero past r
        } else {
            for (int j0 = 0; j0 < r; j0 += 8) {
                const u16x8_t bv = *(const u16x8_t *)(a.B + (long)nn * r + j0);
#pragma unroll
                for (int h = 0; h < 8; ++h) lo += tfull[m][j0 + h] * cvt16<BF16>(bv[h]);
            }
        }
        a.y[(long)m * a.N + nn] = to16<BF16>(v + a.sc * lo);
    }
}

template <int BITS, bool BF16, int MB, int RG, int NW, int NB>
__global__ __launch_bounds__(NW * 64) void gemv_fwd_staged_kernel(const FwdArgs a)
{
    gemv_fwd_staged_body<BITS, BF16, MB, RG, NW, NB>(a, (int)blockIdx.x);
}

// several sibling projections in one launch: the workgroup first finds the projection it belongs to
template <int BITS, bool BF16, int MB, int RG, int NW, int NB>
__global__ __launch_bounds__(NW * 64) void gemv_fwd_staged_siblings_kernel(const FwdMulti ma)
{
    int pi = 0;
    while (pi + 1 < ma.count && (int)blockIdx.x >= ma.wg_end[pi]) ++pi;          // wave-uniform
    const FwdArgs a = ma.p[pi];
    gemv_fwd_staged_body<BITS, BF16, MB, RG, NW, NB>(a, (int)blockIdx.x - (pi ? ma.wg_end[pi - 1] : 0));
}

// ------------------------------------------------------------------------------------------------ backward
// Workgroup (cb, sp): weight columns [CB cb, +CB), CB = 16 * CL, rows n of slice sp; wave w takes 32-row chunks
// w, w+4, ...  Lane (wc = lane % 16, q = lane / 16) holds the CL codes of columns CB cb + CL wc .. of rows
// chunk + 8 q + e, e = 0..7.  MFMA number c of a chunk multiplies dY[m, 32 rows] with the codes at column
// CL wc + c of those rows: D_c[m][k = CB cb + CL wc + c].
template <int BITS>
struct BwdShape {
#ifndef QLORA_BW_CL2
#define QLORA_BW_CL2 16
#endif
#ifndef QLORA_BW_CL4
#define QLORA_BW_CL4 8
#endif
    static constexpr int CL = BITS == 3 ? 32 : (BITS == 2 ? QLORA_BW_CL2 : (BITS == 4 ? QLORA_BW_CL4 : 8));   // columns per lane
    static constexpr int WORDS = CL * BITS / 32;
    static constexpr int CB = 16 * CL;
};


struct BwdArgs {
    const uint16_t *dy;
    const uint32_t *packed;
    const uint16_t *scales;
    const uint8_t *zeros;
    const uint16_t *B;
    float *partial;       // [slices][M][K]
    float *upartial;      // [slices][16][64]
    int M, N, K, r, ng, rows_per_slice;
    uint32_t magic;
};

// code c (compile-time) of a lane's CL codes held in WORDS words
template <int BITS, int WORDS>
__device__ __forceinline__ uint32_t code_of(const uint32_t (&w)[WORDS], int c)
{
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int o = BITS * c, wi = o >> 5, sh = o & 31;
    uint32_t v = w[wi] >> sh;
    if (sh + BITS > 32) v |= w[wi + 1] << (32 - sh);
    return v & mask;
}

// fp16: column c of eight consecutive weight rows as one MFMA fragment (element e = row e).  Rows are handled in
// pairs: one byte permute drops the code of both rows into the mantissas of (1024.0, 1024.0), at bit p of each
// half; a packed fma with (2^-p, -(1024 * 2^-p + z)) leaves the exact integers q - z and a packed multiply applies
// the two rows' scales, so every weight is rounded once from its exact value.
template <int BITS, int WORDS>
__device__ __forceinline__ u16x8_t dequant_rows8_f16(const uint32_t (&w)[8][WORDS], int c, const half2_t (&s2)[4],
                                                     const half2_t (&nz2)[4])
{
    const int o = BITS * c, wi = o >> 5, sh = o & 31;
    const bool straddle = sh + BITS > 32;                 // the code runs into the next word (3-bit codes only)
    const int bb = straddle ? 0 : (sh >> 3), p = straddle ? 0 : (sh & 7);
    const bool two = p + BITS > 8;                        // ... or into the next byte
    const uint32_t sel = (uint32_t)bb | ((two ? (uint32_t)(bb + 1) : 0x0Cu) << 8) | ((uint32_t)(4 + bb) << 16) |
                         ((two ? (uint32_t)(5 + bb) : 0x0Cu) << 24);
    const uint32_t m1 = ((1u << BITS) - 1u) << p, mask2 = m1 | (m1 << 16);
    const half_t mulv = (half_t)(1.f / (float)(1 << p)), offc = (half_t)(-1024.f / (float)(1 << p));
    const half2_t mul2 = {mulv, mulv}, off2 = {offc, offc};
    u32x4_t out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        uint32_t lo = w[2 * i][wi], hi = w[2 * i + 1][wi];
        if (straddle) {
            lo = __builtin_amdgcn_alignbit(w[2 * i][wi + 1 < WORDS ? wi + 1 : wi], lo, (uint32_t)sh);
            hi = __builtin_amdgcn_alignbit(w[2 * i + 1][wi + 1 < WORDS ? wi + 1 : wi], hi, (uint32_t)sh);
        }
        const uint32_t bits = (__builtin_amdgcn_perm(hi, lo, sel) & mask2) | 0x64006400u;
        const half2_t h = __builtin_bit_cast(half2_t, bits);
        out[i] = __builtin_bit_cast(uint32_t, (h * mul2 + (nz2[i] + off2)) * s2[i]);
    }
    return __builtin_bit_cast(u16x8_t, out);
}

// sp_local: row slice inside the projection; sp: slice among all slices of the launch (where its partial sums go)
template <int BITS, bool BF16, int NW, int BW_U>   // NW waves; BW_U 32-row chunks per wave in flight together
__device__ __forceinline__ void gemv_bwd_body(const BwdArgs &a, const int sp_local, const int sp)
{
    using S = BwdShape<BITS>;
    constexpr int CL = S::CL, WORDS = S::WORDS, CB = S::CB;
    constexpr int NT = NW * 64;
    __shared__ float red[NW][16][128 + 1];   // the column block is reduced 128 columns at a time
    __shared__ float ured[NW][16][64 + 1];
    __shared__ uint16_t sz_s[NW][32];        // per wave: scales of its 32 rows (this lane's group is fetched by lane row)
    __shared__ uint8_t sz_z[NW][32];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wc = lane & 15, q = lane >> 4;
    const int N = a.N, K = a.K, r = a.r;
    // Workgroups are dealt to the 8 dies round-robin by their linear index.  A 64-byte piece of a weight row is half
    // a cache line: neighbouring column blocks go to the same die, so that the line is fetched into one L2 only.
    const int ncb = (int)gridDim.x, die = (int)blockIdx.x & 7;
    const int cb = die * (ncb >> 3) + min(die, ncb & 7) + ((int)blockIdx.x >> 3);
    const int kcol = cb * CB + CL * wc;                     // first of this lane's CL columns (all in one group: CL | 32)
    const bool kok = kcol < K;
    const int kc = kok ? kcol : 0;
    const int Kw = K * BITS / 32;
    const int g = group_of(kc, a.magic);
    const int g_block = group_of(cb * CB, a.magic);        // group of the block's first column (lanes past K hold g of column 0)
    const bool uniform_group = g_block == group_of(min(cb * CB + CB, K) - 1, a.magic);
    const int nbeg = sp_local * a.rows_per_slice, nend = min(N, nbeg + a.rows_per_slice);
    const bool do_u = cb == 0 && r > 0;

    float4_t acc[CL], uacc[4];
#pragma unroll
    for (int c = 0; c < CL; ++c) acc[c] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int gg = 0; gg < 4; ++gg) uacc[gg] = float4_t{0.f, 0.f, 0.f, 0.f};

    // A wave's chunks are fetched BW_U at a time before any of them is used: the pass is a handful of dependent
    // memory round trips long, so every load that can be in flight together must be.
    for (int nb = nbeg + wave * 32; nb < nend; nb += 32 * NW * BW_U) {
        uint32_t w[BW_U][8][WORDS];
        u16x8_t df[BW_U], bfr[BW_U][4];        // bfr: B^T fragments for u = dY B (first column block only)
#pragma unroll
        for (int u = 0; u < BW_U; ++u)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg) bfr[u][gg] = ZERO8;
        uint16_t sraw[BW_U][8];
        uint8_t zraw[BW_U][8];
        const int mrow = min(wc, a.M - 1);                    // dY fragment: token row wc, 8 consecutive rows n
#pragma unroll
        for (int u = 0; u < BW_U; ++u) {
            const int n0 = nb + 32 * NW * u;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int nc = min(n0 + 8 * q + e, N - 1);
                const uint32_t *src = a.packed + (long)nc * Kw + (kc / CL) * WORDS;
                if constexpr (WORDS == 2) {
                    const u32x2_t v = *(const u32x2_t *)src;
                    w[u][e][0] = v[0];
                    w[u][e][1] = v[1];
                } else {
#pragma unroll
                    for (int i = 0; i < WORDS; ++i) w[u][e][i] = src[i];
                }
            }
            const int nn = n0 + 8 * q;
            df[u] = *(const u16x8_t *)(a.dy + (long)mrow * N + (nn < nend ? nn : 0));
            if (do_u) {     // gathered column-wise, in flight together with the packed words
#pragma unroll
                for (int gg = 0; gg < 4; ++gg) {
                    const int j = gg * 16 + wc;
                    if (nn < nend && j < r) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) bfr[u][gg][e] = a.B[(long)(nn + e) * r + j];
                    }
                }
            }
            if (uniform_group) {
                // one scale / zero-point per row for the whole column block: lane l < 32 fetches row n0 + l
                const long gi = (long)min(n0 + (lane & 31), N - 1) * a.ng + g_block;
                sraw[u][0] = a.scales[gi];
                zraw[u][0] = a.zeros[gi];
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const long gi = (long)min(n0 + 8 * q + e, N - 1) * a.ng + g;
                    sraw[u][e] = a.scales[gi];
                    zraw[u][e] = a.zeros[gi];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < BW_U; ++u) {
            const int n0 = nb + 32 * NW * u, nn = n0 + 8 * q;
            const bool in = nn < nend;                        // N % 8 == 0, slices are multiples of 32: all or nothing
            const u16x8_t dfu = in ? df[u] : ZERO8;
            float s[8], z[8];
            if (uniform_group) {
                // hand the 32 rows' values round through LDS (wave-private; LDS operations of a wave complete in order)
                if (lane < 32) {
                    sz_s[wave][lane] = sraw[u][0];
                    sz_z[wave][lane] = zraw[u][0];
                }
                __builtin_amdgcn_wave_barrier();
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool ok = kok && n0 + 8 * q + e < nend;
                    s[e] = ok ? f16_bits_to_f32(sz_s[wave][8 * q + e]) : 0.f;
                    z[e] = (float)sz_z[wave][8 * q + e];
                }
                __builtin_amdgcn_wave_barrier();
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const bool ok = kok && n0 + 8 * q + e < nend;
                    s[e] = ok ? f16_bits_to_f32(sraw[u][e]) : 0.f;
                    z[e] = (float)zraw[u][e];
                }
            }
            if (do_u) {     // u = dY B over this chunk
#pragma unroll
                for (int gg = 0; gg < 4; ++gg)
                    if (gg * 16 < r) uacc[gg] = mfma16<BF16>(dfu, bfr[u][gg], uacc[gg]);      // D[m = 4q+v][j = 16 gg + wc]
            }
            if constexpr (BF16) {
#pragma unroll
                for (int c = 0; c < CL; ++c) {
                    u16x8_t wf;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        wf[e] = to16<BF16>(((float)code_of<BITS, WORDS>(w[u][e], c) - z[e]) * s[e]);
                    acc[c] = mfma16<BF16>(dfu, wf, acc[c]);              // D[m = 4q+v][column CL wc + c]
                }
            } else {
                half2_t s2[4], nz2[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    s2[i] = half2_t{(half_t)s[2 * i], (half_t)s[2 * i + 1]};          // exact: they were fp16
                    nz2[i] = half2_t{(half_t)(-z[2 * i]), (half_t)(-z[2 * i + 1])};
                }
#pragma unroll
                for (int c = 0; c < CL; ++c)
                    acc[c] = mfma16<BF16>(dfu, dequant_rows8_f16<BITS, WORDS>(w[u], c, s2, nz2), acc[c]);
            }
        }
    }
    if (do_u) {
#pragma unroll
        for (int gg = 0; gg < 4; ++gg)
#pragma unroll
            for (int v = 0; v < 4; ++v) ured[wave][4 * q + v][16 * gg + wc] = uacc[gg][v];
    }
    for (int cp = 0; cp < CB / 128; ++cp) {
        if (cp) __syncthreads();
        if ((CL * wc) / 128 == cp) {
#pragma unroll
            for (int c = 0; c < CL; ++c)
#pragma unroll
                for (int v = 0; v < 4; ++v) red[wave][4 * q + v][(CL * wc + c) & 127] = acc[c][v];
        }
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * 128; e += NT) {
            const int m = e >> 7, kl = e & 127, k = cb * CB + cp * 128 + kl;
            if (m >= a.M || k >= K) continue;
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) v += red[w][m][kl];
            a.partial[((long)sp * a.M + m) * K + k] = v;
        }
    }
    if (do_u) {
        for (int e = threadIdx.x; e < 16 * 64; e += NT) {
            const int m = e >> 6, j = e & 63;
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) v += ured[w][m][j];
            a.upartial[(long)sp * 1024 + e] = v;
        }
    }
}

struct BwdMulti {
    BwdArgs p[MAX_SIBLINGS];
    int slice_end[MAX_SIBLINGS];      // projection i owns the slices [slice_end[i-1], slice_end[i])
    int count;
};

template <int BITS, bool BF16, int NW, int BW_U>
__global__ __launch_bounds__(NW * 64) void gemv_bwd_kernel(const BwdArgs a)
{
    gemv_bwd_body<BITS, BF16, NW, BW_U>(a, (int)blockIdx.y, (int)blockIdx.y);
}

// sibling projections (same x, so their dX add up): the slices of all of them in one launch
template <int BITS, bool BF16, int NW, int BW_U>
__global__ __launch_bounds__(NW * 64) void gemv_bwd_siblings_kernel(const BwdMulti ma)
{
    const int sp = (int)blockIdx.y;
    int pi = 0;
    while (pi + 1 < ma.count && sp >= ma.slice_end[pi]) ++pi;      // wave-uniform
    const BwdArgs a = ma.p[pi];
    gemv_bwd_body<BITS, BF16, NW, BW_U>(a, sp - (pi ? ma.slice_end[pi - 1] : 0), sp);
}

// Second backward kernel (M <= 16), one thread per output element:
//   blocks [0, xb)        dX[m,k] = sum over slices of partial + sc * sum_j u[m,j] A[j,k]
//   blocks [xb, xb+ab)    dA[j,k] = sc * sum_m u[m,j] x[m,k]
//   blocks [xb+ab, ...)   dB[n,j] = sc * sum_m dY[m,n] t[m,j]
// u = sum over slices of the partial u; every block that needs it sums the few entries itself.
struct FinishArgs {
    const float *partial, *upartial;
    const uint16_t *A, *x, *dy, *t;
    uint16_t *dx;
    float *dA, *dB;
    int M, N, K, r, slices, xb, ab;
    float sc;
};

template <bool BF16>
__global__ __launch_bounds__(256) void gemv_bwd_finish_kernel(const FinishArgs a)
{
    __shared__ float side[16][64 + 1];       // u (dX and dA blocks) or t (dB blocks), as the 16-bit values they round to
    const int M = a.M, r = a.r, K = a.K, N = a.N;
    const int b = blockIdx.x;
    if (b < a.xb + a.ab) {
        for (int e = threadIdx.x; e < M * r; e += 256) {
            const int m = e / r, j = e % r;
            const float *up = a.upartial + m * 64 + j;
            float v = 0.f;
            for (int s0 = 0; s0 < a.slices; s0 += 8) {       // eight slices requested together, summed in slice order
                float pv[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) pv[i] = s0 + i < a.slices ? up[(long)(s0 + i) * 1024] : 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) v += pv[i];
            }
            side[m][j] = cvt16<BF16>(to16<BF16>(v));
        }
    } else {
        for (int e = threadIdx.x; e < M * r; e += 256) side[e / r][e % r] = cvt16<BF16>(a.t[e]);
    }
    __syncthreads();
    if (b < a.xb) {
        const long idx = (long)b * 256 + threadIdx.x;
        if (idx >= (long)M * K) return;
        const int m = (int)(idx / K), k = (int)(idx % K);
        const long stride = (long)M * K;
        float v = 0.f;
        int s = 0;
        for (; s + 4 <= a.slices; s += 4) {
            const float p0 = a.partial[(s + 0) * stride + idx], p1 = a.partial[(s + 1) * stride + idx];
            const float p2 = a.partial[(s + 2) * stride + idx], p3 = a.partial[(s + 3) * stride + idx];
            v = (((v + p0) + p1) + p2) + p3;
        }
        for (; s < a.slices; ++s) v += a.partial[s * stride + idx];
        float lo = 0.f;
        for (int j = 0; j < r; ++j) lo += side[m][j] * cvt16<BF16>(a.A[(long)j * K + k]);
        a.dx[idx] = to16<BF16>(v + a.sc * lo);
    } else if (b < a.xb + a.ab) {
        const long idx = (long)(b - a.xb) * 256 + threadIdx.x;
        if (idx >= (long)r * K) return;
        const int j = (int)(idx / K), k = (int)(idx % K);
        float v = 0.f;
        for (int m = 0; m < M; ++m) v += side[m][j] * cvt16<BF16>(a.x[(long)m * K + k]);
        a.dA[idx] = a.sc * v;
    } else {
        const long idx = (long)(b - a.xb - a.ab) * 256 + threadIdx.x;
        if (idx >= (long)r * N) return;
        const int j = (int)(idx / N), n = (int)(idx % N);
        float v = 0.f;
        for (int m = 0; m < M; ++m) v += cvt16<BF16>(a.dy[(long)m * N + n]) * side[m][j];
        a.dB[(long)n * r + j] = a.sc * v;
    }
}

// The same for sibling projections: dX sums the slices of all of them and every projection's sc * u_i A_i.
//   blocks [0, xb)                 dX
//   blocks [xb, xb + count*ab)     dA of projection (b - xb) / ab
//   then, per projection           dB (its block range ends at bb_end)
struct FinishProj {
    const uint16_t *A, *dy, *t;
    float *dA, *dB;
    int N, slice_begin, slice_end, bb_end;
};
struct FinishMulti {
    FinishProj p[MAX_SIBLINGS];
    const float *partial, *upartial;
    const uint16_t *x;
    uint16_t *dx;
    int M, K, r, slices, xb, ab, count;
    float sc;
};

template <bool BF16>
__global__ __launch_bounds__(256) void gemv_bwd_finish_siblings_kernel(const FinishMulti a)
{
    __shared__ float side[MAX_SIBLINGS][16][64 + 1];
    const int M = a.M, r = a.r, K = a.K;
    const int b = blockIdx.x;
    // u of projection i, as the 16-bit values it rounds to, into side[slot]
    auto sum_u = [&](int i, int slot) {
        const int sb = a.p[i].slice_begin, se = a.p[i].slice_end;
        for (int e = threadIdx.x; e < M * r; e += 256) {
            const int m = e / r, j = e % r;
            const float *up = a.upartial + m * 64 + j;
            float v = 0.f;
            for (int s0 = sb; s0 < se; s0 += 8) {
                float pv[8];
#pragma unroll
                for (int i8 = 0; i8 < 8; ++i8) pv[i8] = s0 + i8 < se ? up[(long)(s0 + i8) * 1024] : 0.f;
#pragma unroll
                for (int i8 = 0; i8 < 8; ++i8) v += pv[i8];
            }
            side[slot][m][j] = cvt16<BF16>(to16<BF16>(v));
        }
    };
    if (b < a.xb) {
        for (int i = 0; i < a.count; ++i) sum_u(i, i);
        __syncthreads();
        const long idx = (long)b * 256 + threadIdx.x;
        if (idx >= (long)M * K) return;
        const int m = (int)(idx / K), k = (int)(idx % K);
        const long stride = (long)M * K;
        float v = 0.f;
        int s = 0;
        for (; s + 4 <= a.slices; s += 4) {
            const float p0 = a.partial[(s + 0) * stride + idx], p1 = a.partial[(s + 1) * stride + idx];
            const float p2 = a.partial[(s + 2) * stride + idx], p3 = a.partial[(s + 3) * stride + idx];
            v = (((v + p0) + p1) + p2) + p3;
        }
        for (; s < a.slices; ++s) v += a.partial[s * stride + idx];
        float lo = 0.f;
        for (int i = 0; i < a.count; ++i)
            for (int j = 0; j < r; ++j) lo += side[i][m][j] * cvt16<BF16>(a.p[i].A[(long)j * K + k]);
        a.dx[idx] = to16<BF16>(v + a.sc * lo);
    } else if (b < a.xb + a.count * a.ab) {
        const int i = (b - a.xb) / a.ab;
        sum_u(i, 0);
        __syncthreads();
        const long idx = (long)((b - a.xb) % a.ab) * 256 + threadIdx.x;
        if (idx >= (long)r * K) return;
        const int j = (int)(idx / K), k = (int)(idx % K);
        float v = 0.f;
        for (int m = 0; m < M; ++m) v += side[0][m][j] * cvt16<BF16>(a.x[(long)m * K + k]);
        a.p[i].dA[idx] = a.sc * v;
    } else {
        const int bb = b - a.xb - a.count * a.ab;
        int i = 0;
        while (i + 1 < a.count && bb >= a.p[i].bb_end) ++i;
        const FinishProj pr = a.p[i];
        for (int e = threadIdx.x; e < M * r; e += 256) side[0][e / r][e % r] = cvt16<BF16>(pr.t[e]);
        __syncthreads();
        const long idx = (long)(bb - (i ? a.p[i - 1].bb_end : 0)) * 256 + threadIdx.x;
        if (idx >= (long)r * pr.N) return;
        const int j = (int)(idx / pr.N), n = (int)(idx % pr.N);
        float v = 0.f;
        for (int m = 0; m < M; ++m) v += cvt16<BF16>(pr.dy[(long)m * pr.N + n]) * side[0][m][j];
        pr.dB[(long)n * r + j] = a.sc * v;
    }
}

inline uint32_t group_magic(int G)
{
    const uint32_t d = (uint32_t)(G / 32);
    return d == 1 ? 0u : (uint32_t)(0x100000000ull / d) + 1u;
}

template <int BITS, bool BF16, int MB>
void launch_fwd_rg(const FwdArgs &a, int rg, hipStream_t s)
{
    constexpr int NW = 4;
    const dim3 grid((a.N + 15) / 16), block(NW * 64);
    switch (rg) {
    case 0: hipLaunchKernelGGL((gemv_fwd_kernel<BITS, BF16, MB, 0, NW, 1>), grid, block, 0, s, a); break;
    case 1: hipLaunchKernelGGL((gemv_fwd_kernel<BITS, BF16, MB, 1, NW, 1>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((gemv_fwd_kernel<BITS, BF16, MB, 2, NW, 1>), grid, block, 0, s, a); break;
    }
}

inline int blocks16(int N) { return (N + 15) / 16; }

template <int BITS, bool BF16, int MB, int RG, int NW, int NB>
void launch_fwd_staged_one(FwdMulti m, hipStream_t s)
{
    constexpr int lds = NW * 2 * (MB + RG) * ST_BLOCK;            // 128 KB of slices at most
    int wgs = 0;
    for (int i = 0; i < m.count; ++i) {
        wgs += (blocks16(m.p[i].N) + NB - 1) / NB;
        m.wg_end[i] = wgs;
    }
    if (m.count == 1) {
        auto kern = gemv_fwd_staged_kernel<BITS, BF16, MB, RG, NW, NB>;
        static bool configured = false;   // raising the dynamic-LDS ceiling is a property of the function, set once
        if (!configured) {
            (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            configured = true;
        }
        hipLaunchKernelGGL(kern, dim3(wgs), dim3(NW * 64), lds, s, m.p[0]);
        return;
    }
    if constexpr (MB == 1) {          // the callers hand siblings over together only up to 16 token rows
        auto kern = gemv_fwd_staged_siblings_kernel<BITS, BF16, MB, RG, NW, NB>;
        static bool configured = false;
        if (!configured) {
            (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            configured = true;
        }
        hipLaunchKernelGGL(kern, dim3(wgs), dim3(NW * 64), lds, s, m);
    }
}

template <int BITS, bool BF16, int MB, int RG>
void launch_fwd_staged_rg(const FwdMulti &m, hipStream_t s)
{
    // Every workgroup pulls all of x and A through its compute unit once, however many weight rows it owns, and the
    // slices leave room for one workgroup per compute unit: the launch should be a single round of the 256 units.
    // So a workgroup takes as many 16-row blocks (up to four; one token block only: the registers are needed for the
    // packed words) as it takes to get there.  Siblings that do not fit one round together go out one by one.
    constexpr int NW = MB + RG <= 2 ? 8 : 4;
    if constexpr (MB == 1) {
        constexpr int NBMAX = BITS == 8 ? 3 : 4;              // 8-bit words: four blocks' worth would spill
        int nb = 0;
        for (int cand = 1; cand <= NBMAX && nb == 0; ++cand) {
            int wgs = 0;
            for (int i = 0; i < m.count; ++i) wgs += (blocks16(m.p[i].N) + cand - 1) / cand;
            if (wgs <= 256) nb = cand;
        }
        if (nb == 0 && m.count > 1) {
            for (int i = 0; i < m.count; ++i) {
                FwdMulti one{};
                one.count = 1;
                one.p[0] = m.p[i];
                launch_fwd_staged_rg<BITS, BF16, MB, RG>(one, s);
            }
            return;
        }
        switch (nb == 0 ? NBMAX : nb) {
        case 4: launch_fwd_staged_one<BITS, BF16, MB, RG, NW, NBMAX>(m, s); return;
        case 3: launch_fwd_staged_one<BITS, BF16, MB, RG, NW, 3>(m, s); return;
        case 2: launch_fwd_staged_one<BITS, BF16, MB, RG, NW, 2>(m, s); return;
        default: break;
        }
    }
    launch_fwd_staged_one<BITS, BF16, MB, RG, NW, 1>(m, s);
}

template <int BITS, bool BF16, int MB>
void launch_fwd_staged(const FwdMulti &m, int rg, hipStream_t s)
{
    switch (rg) {
    case 0: launch_fwd_staged_rg<BITS, BF16, MB, 0>(m, s); break;
    case 1: launch_fwd_staged_rg<BITS, BF16, MB, 1>(m, s); break;
    default: launch_fwd_staged_rg<BITS, BF16, MB, 2>(m, s); break;
    }
}

template <int BITS, bool BF16>
void launch_fwd_mb(const FwdMulti &m, int rg, hipStream_t s)
{
    switch ((m.p[0].M + 15) / 16) {
    case 1: launch_fwd_staged<BITS, BF16, 1>(m, rg, s); break;
    case 2:
        for (int i = 0; i < m.count; ++i) {
            FwdMulti one{};
            one.count = 1;
            one.p[0] = m.p[i];
            launch_fwd_staged<BITS, BF16, 2>(one, rg, s);
        }
        break;
    case 3:
        for (int i = 0; i < m.count; ++i) launch_fwd_rg<BITS, BF16, 3>(m.p[i], rg, s);
        break;
    default:
        for (int i = 0; i < m.count; ++i) launch_fwd_rg<BITS, BF16, 4>(m.p[i], rg, s);
        break;
    }
}

template <int BITS, bool BF16>
void launch_bwd_bits(const BwdMulti &m, hipStream_t s)
{
    const int slices = m.slice_end[m.count - 1];
    int max_rows = 0;
    for (int i = 0; i < m.count; ++i) max_rows = m.p[i].rows_per_slice > max_rows ? m.p[i].rows_per_slice : max_rows;
    const dim3 grid((m.p[0].K + BwdShape<BITS>::CB - 1) / BwdShape<BITS>::CB, slices);
    // Two chunks per wave in flight (more would not fit the register file at eight waves); eight waves share out the
    // arithmetic of a slice, four are enough when the slice has no more than eight chunks.
    bool eight = false;
    if constexpr (BITS != 3) eight = max_rows / 32 > 8;   // 3-bit: 32 columns per lane, the accumulators need the four-wave register budget
    if (m.count == 1) {
        if constexpr (BITS != 3) {
            if (eight) {
                hipLaunchKernelGGL((gemv_bwd_kernel<BITS, BF16, 8, 2>), grid, dim3(512), 0, s, m.p[0]);
                return;
            }
        }
        hipLaunchKernelGGL((gemv_bwd_kernel<BITS, BF16, 4, 2>), grid, dim3(256), 0, s, m.p[0]);
        return;
    }
    if constexpr (BITS != 3) {
        if (eight) {
            hipLaunchKernelGGL((gemv_bwd_siblings_kernel<BITS, BF16, 8, 2>), grid, dim3(512), 0, s, m);
            return;
        }
    }
    hipLaunchKernelGGL((gemv_bwd_siblings_kernel<BITS, BF16, 4, 2>), grid, dim3(256), 0, s, m);
}

int bwd_cb(int bits) { return bits == 3 ? BwdShape<3>::CB : (bits == 2 ? BwdShape<2>::CB : (bits == 4 ? BwdShape<4>::CB : BwdShape<8>::CB)); }

}  // namespace

int gemv_bwd_slices(int N, int K, int bits)
{
    const int colblocks = (K + bwd_cb(bits) - 1) / bwd_cb(bits);
    int slices = (256 + colblocks - 1) / colblocks;      // aim at one workgroup per compute unit: every extra slice
                                                         // costs another M x K block of partial sums
    const int max_slices = (N + 127) / 128;              // at least four 32-row chunks per workgroup
    if (slices > max_slices) slices = max_slices;
    return slices < 1 ? 1 : slices;
}

int gemv_bwd_slices_siblings(int count, const int *N, int K, int bits, int *slices)
{
    if (count == 1) {
        slices[0] = gemv_bwd_slices(N[0], K, bits);
        return slices[0];
    }
    const int colblocks = (K + bwd_cb(bits) - 1) / bwd_cb(bits);
    const int target = (256 + colblocks - 1) / colblocks;
    long rows = 0;
    for (int i = 0; i < count; ++i) rows += N[i];
    int total = 0;
    for (int i = 0; i < count; ++i) {       // the launch's slices are shared out in proportion to the rows
        int sl = (int)(((long)target * N[i] + rows / 2) / rows);
        const int max_slices = (N[i] + 127) / 128;
        if (sl > max_slices) sl = max_slices;
        if (sl < 1) sl = 1;
        slices[i] = sl;
        total += sl;
    }
    while (total > target) {                // rounding must not push the launch into a second round of workgroups
        int big = 0;
        for (int i = 1; i < count; ++i)
            if ((long)slices[i] * N[big] > (long)slices[big] * N[i] || (slices[big] == 1 && slices[i] > 1)) big = i;
        if (slices[big] == 1) break;        // one slice each is the least there is
        --slices[big];
        --total;
    }
    return total;
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

bool fwd_small_computes_t(int rank) { return rank > 0 && rank <= 32; }

void launch_fwd_small(const Problem &p, int count, const void *x, const uint32_t *const *packed,
                      const void *const *scales, const uint8_t *const *zeros, const void *const *A,
                      const void *const *B, const void *const *t_in, void *const *t_out, void *const *y, const int *N,
                      hipStream_t s)
{
    const bool fused = fwd_small_computes_t(p.r);
    FwdMulti m{};
    m.count = count;
    for (int i = 0; i < count; ++i)
        m.p[i] = FwdArgs{(const uint16_t *)x,
                         packed[i],
                         (const uint16_t *)scales[i],
                         zeros[i],
                         (const uint16_t *)(A ? A[i] : nullptr),
                         (const uint16_t *)(B ? B[i] : nullptr),
                         fused ? nullptr : (const uint16_t *)(t_in ? t_in[i] : nullptr),
                         (uint16_t *)y[i],
                         fused ? (uint16_t *)(t_out ? t_out[i] : nullptr) : nullptr,
                         p.M,
                         N[i],
                         p.K,
                         p.r,
                         p.K / p.G,
                         p.sc,
                         group_magic(p.G)};
    const int rg = fused ? (p.r + 15) / 16 : 0;
    QLORA_BITS_DTYPE(launch_fwd_mb, m, rg, s);
}

void launch_bwd_small(const Problem &p, int count, const void *const *dy, const void *x,
                      const uint32_t *const *packed, const void *const *scales, const uint8_t *const *zeros,
                      const void *const *A, const void *const *B, const void *const *t, void *dx, float *const *dA,
                      float *const *dB, const int *N, float *partial, float *upartial, hipStream_t s)
{
    int slices[MAX_SIBLINGS];
    const int total = gemv_bwd_slices_siblings(count, N, p.K, p.bits, slices);
    BwdMulti m{};
    m.count = count;
    int end = 0;
    for (int i = 0; i < count; ++i) {
        const int rows_per_slice = ((N[i] + slices[i] - 1) / slices[i] + 31) / 32 * 32;
        m.p[i] = BwdArgs{(const uint16_t *)dy[i], packed[i], (const uint16_t *)scales[i], zeros[i],
                         (const uint16_t *)(B ? B[i] : nullptr), partial, upartial, p.M, N[i], p.K, p.r, p.K / p.G,
                         rows_per_slice, group_magic(p.G)};
        end += slices[i];
        m.slice_end[i] = end;
    }
    QLORA_BITS_DTYPE(launch_bwd_bits, m, s);
    const int xb = (int)(((long)p.M * p.K + 255) / 256), ab = (int)(((long)p.r * p.K + 255) / 256);
    if (count == 1) {
        const int bb = (int)(((long)p.r * N[0] + 255) / 256);
        const FinishArgs f{partial, upartial, (const uint16_t *)(A ? A[0] : nullptr), (const uint16_t *)x,
                           (const uint16_t *)dy[0], (const uint16_t *)(t ? t[0] : nullptr), (uint16_t *)dx,
                           dA ? dA[0] : nullptr, dB ? dB[0] : nullptr, p.M, N[0], p.K, p.r, total, xb, ab, p.sc};
        if (p.bf16)
            hipLaunchKernelGGL((gemv_bwd_finish_kernel<true>), dim3(xb + ab + bb), dim3(256), 0, s, f);
        else
            hipLaunchKernelGGL((gemv_bwd_finish_kernel<false>), dim3(xb + ab + bb), dim3(256), 0, s, f);
        return;
    }
    FinishMulti f{};
    f.partial = partial;
    f.upartial = upartial;
    f.x = (const uint16_t *)x;
    f.dx = (uint16_t *)dx;
    f.M = p.M;
    f.K = p.K;
    f.r = p.r;
    f.slices = total;
    f.xb = xb;
    f.ab = ab;
    f.count = count;
    f.sc = p.sc;
    int bb_end = 0, sb = 0;
    for (int i = 0; i < count; ++i) {
        bb_end += (int)(((long)p.r * N[i] + 255) / 256);
        f.p[i] = FinishProj{(const uint16_t *)(A ? A[i] : nullptr), (const uint16_t *)dy[i],
                            (const uint16_t *)(t ? t[i] : nullptr), dA ? dA[i] : nullptr, dB ? dB[i] : nullptr,
                            N[i], sb, sb + slices[i], bb_end};
        sb += slices[i];
    }
    const int blocks = xb + count * ab + bb_end;
    if (p.bf16)
        hipLaunchKernelGGL((gemv_bwd_finish_siblings_kernel<true>), dim3(blocks), dim3(256), 0, s, f);
    else
        hipLaunchKernelGGL((gemv_bwd_finish_siblings_kernel<false>), dim3(blocks), dim3(256), 0, s, f);
}

}  // namespace qlora
