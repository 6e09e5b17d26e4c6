// Small-token-count forward kernels and their launchers, as a header: one translation unit per code width
// (gemv_fwd_b2.hip ... gemv_fwd_b8.hip) instantiates them, so that the widths compile in parallel.
#pragma once
#include "gemv_common.hpp"


namespace qlora {

namespace {

// ------------------------------------------------------------------------------------------------- forward
// LDS slice of one 16-row block: 16 rows x 16 pieces of 16 bytes; piece c of row w sits in slot 16 w + (c ^ w), so
// the fragment reads of 16 rows at one piece index fall on 16 different bank groups.
constexpr int ST_BLOCK = 4096;      // bytes of one 16-row x 128-column block
constexpr int ST_U = 4;             // iterations whose packed words are requested together
static_assert(ST_U % 2 == 0, "a batch starts on slice buffer 0: the buffer of iteration i0 + u is u & 1");

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
        ensure_dynamic_lds((const void *)kern, (int)(lds));
        QLORA_LAUNCH(kern, dim3(wgs), dim3(NW * 64), lds, s, m.p[0]);
        return;
    }
    if constexpr (MB == 1) {          // the callers hand siblings over together only up to 16 token rows
        auto kern = gemv_fwd_staged_siblings_kernel<BITS, BF16, MB, RG, NW, NB>;
        ensure_dynamic_lds((const void *)kern, (int)(lds));
        QLORA_LAUNCH(kern, dim3(wgs), dim3(NW * 64), lds, s, m);
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

}  // namespace

}  // namespace qlora

#include "gemv_fwd_m16.hpp"

namespace qlora {

namespace {

template <int BITS, bool BF16>
bool launch_fwd_mb(const FwdMulti &m, int rg, hipStream_t s)
{
    const bool zpacked = m.p[0].zpacked != nullptr;       // only the kernel with staged group constants reads those
    if (launch_fwd_m16<BITS, BF16>(m, rg, s)) return true;
    if (zpacked) return false;
    if (m.p[0].M <= 16) {
        launch_fwd_staged<BITS, BF16, 1>(m, rg, s);
    } else {                                              // up to SMALL_M_FWD_MAX = 32 rows
        for (int i = 0; i < m.count; ++i) {
            FwdMulti one{};
            one.count = 1;
            one.p[0] = m.p[i];
            launch_fwd_staged<BITS, BF16, 2>(one, rg, s);
        }
    }
    return true;
}

}  // namespace

template <int BITS>
bool launch_fwd_small_bits(const FwdMulti &m, int rg, bool bf16, hipStream_t s)
{
    return bf16 ? launch_fwd_mb<BITS, true>(m, rg, s) : launch_fwd_mb<BITS, false>(m, rg, s);
}

}  // namespace qlora
