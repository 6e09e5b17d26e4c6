// Forward pass for up to 32 token rows (one or two 16-row token blocks) with the packed weight staged through LDS
// (included by gemv_fwd_impl.hpp).
//
// What bounds the pass at this size is the number of memory instructions and cache lines a compute unit has to work
// through, not the bytes: a lane that fetches its own MFMA fragment of a 2-bit weight touches 8 bytes of a row, so a
// wave instruction brings in sixteen 32-byte pieces, and the group constants cost two more such instructions per
// fragment.  Here nothing is fetched fragment-wise.  A workgroup of eight waves owns 16 NB weight rows and walks K in
// stages of 8 KS columns (KS = 128; 64 for 8-bit codes, for two token blocks and for 32 adapter rows): per stage the
// packed words of all its rows (row segments of KS BITS bytes, whole cache lines), the token rows of x (16 or 32; only
// the requests that hold rows below M are made) and the adapter rows of A arrive by direct-to-LDS loads of 1 KB per
// instruction, two stages in flight, and every wave takes the fragments of its KS contraction indices from LDS.  The
// group constants of all the workgroup's rows are copied to LDS once, at the start.
//
// Layout of a stage in LDS: per wave a slice of x (16 MB rows x KS columns) and an AR-row slice of A (piece c of row
// w in slot (KS / 8) w + (c ^ w mod KS / 8), as in the staged kernel); then the weight chunk, row n at n * KS BITS
// bytes, its 16-byte pieces permuted by wswz() so that sixteen rows read at one piece index fall on different banks.
#pragma once

namespace qlora {

namespace {

constexpr int M16_NW = 8;                  // waves of a workgroup; wave w owns columns KS w .. KS w + KS of a stage
constexpr int M16_LDS = 160 * 1024;
// Columns of a wave per stage and stages in LDS.  8-bit codes: half the columns, so that three blocks of weight rows
// fit beside the activations, and three stages (one barrier per stage instead of two).  The narrower widths are
// faster with the wide slices (INT2 gate/up at M = 16: 12.0 against 13.3 us).
// With two 16-row token blocks (mb = 2: 17 to 32 token rows) the slices are 64 columns wide for every code width, so
// that 32 rows of x per wave fit, and there are two stages.
// The same narrow slices when 32 rows of A ride along (ranks 17 to 32).
constexpr int m16_ks(int bits, int mb, int ar) { return bits == 8 || mb == 2 || ar == 32 ? 64 : 128; }
constexpr int m16_nst(int bits, int mb, int ar) { return bits == 8 && mb == 1 && ar <= 16 ? 3 : 2; }

// slot of the 16-byte piece `piece` of weight row n inside the row's stage segment of PPR pieces (its own inverse)
template <int BITS, int PPR>
__device__ __forceinline__ int wswz(int n, int piece)
{
    if constexpr (BITS == 3) return 3 * ((piece / 3) ^ (n & 7)) + piece % 3;       // whole units of 12 bytes stay together
    else return piece ^ (n & (PPR < 16 ? PPR - 1 : 15));
}

constexpr int m16_xa(int bits, int ar, int mb) { return (16 * mb + ar) * 2 * m16_ks(bits, mb, ar); }   // a wave's slices of x and A
constexpr int m16_stage(int bits, int nb, int ar, int mb)
{
    return M16_NW * m16_xa(bits, ar, mb) + nb * 16 * m16_ks(bits, mb, ar) * bits;
}
constexpr int m16_table(int nb, int ng, int zrow)     // scales (2 B per group), zero-points (zrow bytes per row: one per
{                                                     // group, or the row's packed words), each filled in whole KB
    return ((nb * 16 * ng * 2 + 1023) & ~1023) + ((nb * 16 * zrow + 1023) & ~1023);
}
constexpr int m16_rga(int ar) { return ar > 16 ? 2 : 1; }                                     // 16-column blocks of t formed here
constexpr int m16_red(int nb, int mb, int ar) { return M16_NW * (nb + m16_rga(ar)) * 16 * mb * 17 * 4; }   // the waves' partial sums
constexpr int m16_tc(int ar) { return ar > 16 ? 32 : (ar > 0 ? 16 : 64); }                    // columns of t kept
constexpr int m16_static(int ar, int mb) { return 16 * mb * (m16_tc(ar) + 1) * 4; }

// s_waitcnt vmcnt(n) for a wave-uniform n in [0, MAX] (the count is an immediate of the instruction)
template <int MAX>
__device__ __forceinline__ void wait_vm_upto(int n)
{
    if constexpr (MAX == 0) {
        wait_vm<0>();
    } else {
        if (n >= MAX) wait_vm<MAX>();
        else wait_vm_upto<MAX - 1>(n);
    }
}

// NB 16-row weight blocks; AR rows of A staged (0: t is given, or no adapter); MB 16-row token blocks (1 or 2)
template <int BITS, bool BF16, int NB, int AR, int MB>
__device__ __forceinline__ void gemv_fwd_m16_body(const FwdArgs &a, const int wg)
{
    constexpr int NW = M16_NW, NT = NW * 64, R = 16 * NB, XROWS = 16 * MB;
    constexpr int KS = m16_ks(BITS, MB, AR), KC = NW * KS, NST = m16_nst(BITS, MB, AR), SS = KS / 32;   // SS: MFMA steps of a wave per stage
    constexpr int PPR = KS * BITS / 16, UB = KS * BITS / 32; // pieces of a weight row per stage; bytes of a lane's codes
    constexpr int PR = KS / 8, RPI = 64 / PR;                // pieces of an activation row per stage; rows per request
    constexpr int XBYTES = 2 * XROWS * KS;                   // a wave's slice of x
    constexpr int XA = m16_xa(BITS, AR, MB), WOFF = NW * XA, STAGE = m16_stage(BITS, NB, AR, MB);
    constexpr int WI = R * PPR / 64;                         // weight requests per stage, dealt out wave by wave
    constexpr int WI_HI = (WI + NW - 1) / NW, WI_LO = WI / NW;
    constexpr int XIX = XROWS / RPI, XIA = AR / RPI, XI = XIX + XIA;   // requests of a wave's own slices
    constexpr int TC = m16_tc(AR), RGA = m16_rga(AR);
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    __shared__ float tfull[XROWS][TC + 1];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, q = lane >> 4;
    const int n0 = wg * R, K = a.K, Kw = K * BITS / 32, r = a.r, ng = a.ng;
    const int rows_here = min(R, a.N - n0);                  // at least one
    const int S = (K + KC - 1) / KC;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;
    const uint16_t *sct = (const uint16_t *)(lds + NST * STAGE);                          // [R][ng], then, from the next
    const uint8_t *zt = lds + NST * STAGE + ((R * ng * 2 + 1023) & ~1023);                // full KB on, the zero-points
    const int zrow = a.zpacked ? a.zw * 4 : ng;                                         // bytes of a row of zero-points

    // ---- this lane's part of the copies.  Weight instruction i of a stage fills slots 64 i .. 64 i + 64 of the chunk.
    const uint32_t *wbase = a.packed + (long)n0 * Kw;
    const uint32_t row_bytes = (uint32_t)Kw * 4u;
    uint32_t w_src[WI_HI], w_piece[WI_HI];                   // byte offset of the row; byte position of the piece in a stage
#pragma unroll
    for (int c = 0; c < WI_HI; ++c) {
        const int e = 64 * (wave + NW * c) + lane, n = min(e / PPR, R - 1), slot = e % PPR;
        w_src[c] = (uint32_t)min(n, rows_here - 1) * row_bytes;
        w_piece[c] = (uint32_t)wswz<BITS, PPR>(n, slot) * 16u;
    }
    // requests that bring in token rows below M (a request moves RPI rows); the rows of x past them are never fetched:
    // what the MFMAs make of the stale LDS there lands in output rows that are not stored
    const int xreq = min(XIX, (a.M + RPI - 1) / RPI);                       // workgroup-uniform
    uint32_t x_src[XIX], a_src[XIA > 0 ? XIA : 1];
#pragma unroll
    for (int j = 0; j < XIX; ++j) {
        const int row = RPI * j + lane / PR, piece = (lane % PR) ^ (row & (PR - 1));
        x_src[j] = (uint32_t)(((long)min(row, a.M - 1) * K + 8 * piece) * 2);
    }
#pragma unroll
    for (int j = 0; j < XIA; ++j) {
        const int row = RPI * j + lane / PR, piece = (lane % PR) ^ (row & (PR - 1));
        a_src[j] = (uint32_t)(((long)min(row, r - 1) * K + 8 * piece) * 2);
    }
    // the requests of one stage, one at a time (they are spread over the arithmetic of the stage before: a request
    // waits for room in the memory pipeline, and meanwhile the wave could be multiplying)
    constexpr int NS = WI_HI + XI;
    auto issue_step = [&](int st, int buf, int j) {
        const uint32_t base = lds0 + (uint32_t)buf * STAGE;
        const int k0 = st * KC + wave * KS;
        const uint32_t kb = k0 < K ? (uint32_t)k0 * 2u : 0u;                 // a slice past K repeats the first one, unused
        if (j < WI_HI) {
            if (wave + NW * j < WI) {                                         // wave-uniform
                const uint32_t at = (uint32_t)st * (uint32_t)(KS * BITS) + w_piece[j];   // the stage's segment of a packed row
                dma16(wbase, w_src[j] + (at < row_bytes ? at : 0u), base + WOFF + (uint32_t)(wave + NW * j) * 1024u);
            }
        } else if (j < WI_HI + XIX) {
            if (j - WI_HI < xreq) dma16(a.x, x_src[j - WI_HI] + kb, base + (uint32_t)wave * XA + (j - WI_HI) * 1024u);
        } else {
            dma16(a.A, a_src[j - WI_HI - XIX] + kb, base + (uint32_t)wave * XA + XBYTES + (j - WI_HI - XIX) * 1024u);
        }
    };
    auto issue = [&](int st, int buf) {
#pragma unroll
        for (int j = 0; j < NS; ++j) issue_step(st, buf, j);
    };
    const bool w_hi = wave < WI - NW * WI_LO;                                 // this wave issues WI_HI weight instructions

    // ---- group constants of all rows of the workgroup: copied as they lie (the rows are neighbours), 1 KB per request;
    //      a piece past the end of the array repeats the array's first one (it belongs to rows past N)
    {
        const uint32_t sbytes = (uint32_t)R * ng * 2u, zbytes = (uint32_t)R * zrow;
        const uint32_t s_all = (uint32_t)a.N * ng * 2u, z_all = (uint32_t)a.N * zrow;
        const uint32_t s0 = (uint32_t)n0 * ng * 2u, z0 = (uint32_t)n0 * zrow;
        const void *zsrc = a.zpacked ? (const void *)a.zpacked : (const void *)a.zeros;
        const uint32_t tb = lds0 + NST * STAGE, zb = tb + ((sbytes + 1023u) & ~1023u);
        for (uint32_t o = (uint32_t)wave * 1024u; o < sbytes; o += NW * 1024u) {
            const uint32_t at = s0 + o + lane * 16u;
            dma16(a.scales, at + 16u <= s_all ? at : 0u, tb + o);
        }
        for (uint32_t o = (uint32_t)wave * 1024u; o < zbytes; o += NW * 1024u) {
            const uint32_t at = z0 + o + lane * 16u;
            dma16(zsrc, at + 16u <= z_all ? at : 0u, zb + o);
        }
    }
    issue(0, 0);
    if (S > 1) issue(1, 1);
    // the rows of B the outputs need at the very end
    constexpr int OPB = 16 * XROWS;                          // outputs per block of weight rows
    constexpr int EPT = (NB * OPB + NT - 1) / NT, BV = AR > 0 ? AR / 8 : 1;
    u16x8_t bpre[EPT][BV];
    if constexpr (AR > 0) {
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int e = threadIdx.x + x * NT, nn = n0 + (e / OPB) * 16 + (e & 15);
            const bool live = e < NB * OPB && nn < a.N;
#pragma unroll
            for (int h = 0; h < BV; ++h)
                bpre[x][h] = (live && 8 * h < r) ? *(const u16x8_t *)(a.B + (long)nn * r + 8 * h) : ZERO8;
        }
    }

    float4_t acc[MB][NB], tacc[MB][RGA];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
        for (int g = 0; g < RGA; ++g) tacc[mb][g] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[mb][nb] = float4_t{0.f, 0.f, 0.f, 0.f};
    }

    for (int st = 0; st < S; ++st) {
        // stage st has landed once at most the requests of stage st + 1 (issued after it) are outstanding
        if (st + 1 < S) {
            wait_vm_upto<WI_HI + XI>((w_hi ? WI_HI : WI_LO) + xreq + XIA);
        } else {
            wait_vm<0>();
        }
        __syncthreads();                                     // ... for every wave; also publishes the group constants
        const int bi = st % NST;
        const uint8_t *buf = lds + (size_t)bi * STAGE;
        const uint8_t *xs = buf + (size_t)wave * XA, *wc = buf + WOFF;
        const int k0 = st * KC + wave * KS;
        const bool live = k0 < K;                            // wave-uniform
        u16x8_t xf[MB][SS], af[RGA][SS];
        uint32_t w[NB][BITS];                                // the first UB bytes are used
        float sc[NB], zp[NB];
#pragma unroll
        for (int s = 0; s < SS; ++s) {
            const int slot = li * PR + ((SS * q + s) ^ (li & (PR - 1)));        // 16 rows on: the same slot key
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) xf[mb][s] = *(const u16x8_t *)(xs + (16 * mb * PR + slot) * 16);
            if constexpr (AR > 0) {
#pragma unroll
                for (int g = 0; g < RGA; ++g)       // adapter rows 16 g + li: 16 rows on, the same slot key
                    af[g][s] = 16 * g + li < min(r, AR) ? *(const u16x8_t *)(xs + XBYTES + (16 * g * PR + slot) * 16) : ZERO8;
            }
        }
        const int grp = live ? group_of(k0, a.magic) : 0;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int n = nb * 16 + li;
            const uint8_t *rowp = wc + n * (PPR * 16);
            if constexpr (BITS == 3) {
                const uint32_t *p = (const uint32_t *)(rowp + (wave ^ (n & 7)) * 48 + 12 * q);
#pragma unroll
                for (int i = 0; i < 3; ++i) w[nb][i] = p[i];
            } else {
                const int ob = (4 * wave + q) * UB;           // the lane's codes inside the row's segment
                if constexpr (UB >= 16) {
#pragma unroll
                    for (int h = 0; h < UB / 16; ++h) {
                        const u32x4_t v = *(const u32x4_t *)(rowp + wswz<BITS, PPR>(n, (ob >> 4) + h) * 16);
#pragma unroll
                        for (int i = 0; i < 4; ++i) w[nb][4 * h + i] = v[i];
                    }
                } else if constexpr (UB == 8) {
                    const u32x2_t v = *(const u32x2_t *)(rowp + wswz<BITS, PPR>(n, ob >> 4) * 16 + (ob & 15));
                    w[nb][0] = v[0];
                    w[nb][1] = v[1];
                } else {
                    w[nb][0] = *(const uint32_t *)(rowp + wswz<BITS, PPR>(n, ob >> 4) * 16 + (ob & 15));
                }
#pragma unroll
                for (int i = UB / 4; i < BITS; ++i) w[nb][i] = 0u;
            }
            sc[nb] = live ? f16_bits_to_f32(sct[n * ng + grp]) : 0.f;
            zp[nb] = a.zpacked ? (float)packed_zero<BITS>((const uint32_t *)(zt + n * zrow), grp) : (float)zt[n * ng + grp];
        }
        wait_lds();                                          // everything of this stage is in registers
        const bool more = st + 2 < S;                        // workgroup-uniform
        const int fill = (st + 2) % NST;                     // two stages: the buffer just read, once every wave is done
        if (NST == 2 && more) __syncthreads();               // with it; three: the one every wave left a step ago
        if (!live) {
            if (more) issue(st + 2, fill);
            continue;
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            // the wave's columns lie in one group: the MFMAs sum x (q - z), exact integers times x, and the
            // scale is applied to the four sums of the lane's weight row
            DequantConst<BITS, BF16> dq;
            dq.set(1.f, zp[nb]);
            float4_t part[MB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) part[mb] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < SS; ++s) {
                if (more && SS * nb + s < NS) issue_step(st + 2, fill, SS * nb + s);
                const u16x8_t wf = dequant8<BITS, BF16, false>(w[nb], s, dq);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) part[mb] = mfma16<BF16>(xf[mb][s], wf, part[mb]);   // D[m = 4q+v][n = li]
            }
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[mb][nb][v] = fmaf(sc[nb], part[mb][v], acc[mb][nb][v]);
        }
        if constexpr (AR > 0) {
#pragma unroll
            for (int s = 0; s < SS; ++s) {
                if (more && SS * NB + s < NS) issue_step(st + 2, fill, SS * NB + s);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int g = 0; g < RGA; ++g) tacc[mb][g] = mfma16<BF16>(xf[mb][s], af[g][s], tacc[mb][g]);   // D[m][j = 16 g + li]
            }
        }
        if (more) {
#pragma unroll
            for (int j = SS * NB + (AR > 0 ? SS : 0); j < NS; ++j) issue_step(st + 2, fill, j);
        }
    }

    // ---- the waves' partial sums meet in LDS (where the stages were)
    __syncthreads();
    float *red = (float *)lds;                               // [NW][NB + RGA][XROWS][17], over the stages and tables
    auto red_at = [&](int w, int blk, int row, int col) -> float & {
        return red[((w * (NB + RGA) + blk) * XROWS + row) * 17 + col];
    };
    static_assert(m16_red(NB, MB, AR) <= M16_LDS - m16_static(AR, MB), "partial sums fit (the launch sizes LDS for them)");
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) red_at(wave, nb, 16 * mb + 4 * q + v, li) = acc[mb][nb][v];
            if constexpr (AR > 0) {
#pragma unroll
                for (int g = 0; g < RGA; ++g) red_at(wave, NB + g, 16 * mb + 4 * q + v, li) = tacc[mb][g][v];
            }
        }
    __syncthreads();
    if constexpr (AR > 0) {
        for (int e = threadIdx.x; e < XROWS * (16 * RGA); e += NT) {
            const int m = e / (16 * RGA), j = e % (16 * RGA);
            float tv = 0.f;
            if (j < r && m < a.M) {
#pragma unroll
                for (int w = 0; w < NW; ++w) tv += red_at(w, NB + (j >> 4), m, j & 15);
                tv = cvt16<BF16>(to16<BF16>(tv));            // the value every consumer of t sees
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
        const int nb = e / OPB, m = (e >> 4) % XROWS, nl = e & 15, nn = n0 + nb * 16 + nl;
        if (e >= NB * OPB || m >= a.M || nn >= a.N) continue;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) v += red_at(w, nb, m, nl);
        float lo = 0.f;
        if constexpr (AR > 0) {
#pragma unroll
            for (int h = 0; h < BV; ++h)
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

template <int BITS, bool BF16, int NB, int AR, int MB>
__global__ __launch_bounds__(M16_NW * 64) void gemv_fwd_m16_kernel(const FwdMulti ma)
{
    int pi = 0;
    while (pi + 1 < ma.count && (int)blockIdx.x >= ma.wg_end[pi]) ++pi;          // wave-uniform
    const FwdArgs a = ma.p[pi];
    gemv_fwd_m16_body<BITS, BF16, NB, AR, MB>(a, (int)blockIdx.x - (pi ? ma.wg_end[pi - 1] : 0));
}

inline int m16_zrow(const FwdArgs &a) { return a.zpacked ? a.zw * 4 : a.ng; }

// largest NB whose stages and tables fit in LDS (0: none)
template <int BITS>
inline int m16_nb_max(int ar, int ng, int zrow, int mb)
{
    for (int nb = 4; nb >= 1; --nb)
        if (m16_nst(BITS, mb, ar) * m16_stage(BITS, nb, ar, mb) + m16_table(nb, ng, zrow) + m16_static(ar, mb) <= M16_LDS)
            return nb;
    return 0;
}

template <int BITS, bool BF16, int NB, int AR, int MB>
void launch_fwd_m16_one(FwdMulti m, hipStream_t s)
{
    const int pipe = m16_nst(BITS, MB, AR) * m16_stage(BITS, NB, AR, MB) + m16_table(NB, m.p[0].ng, m16_zrow(m.p[0]));
    const int lds = pipe > m16_red(NB, MB, AR) ? pipe : m16_red(NB, MB, AR);
    int wgs = 0;
    for (int i = 0; i < m.count; ++i) {
        wgs += (blocks16(m.p[i].N) + NB - 1) / NB;
        m.wg_end[i] = wgs;
    }
    auto kern = gemv_fwd_m16_kernel<BITS, BF16, NB, AR, MB>;
    ensure_dynamic_lds((const void *)kern, M16_LDS - m16_static(AR, MB));
    QLORA_LAUNCH(kern, dim3(wgs), dim3(M16_NW * 64), lds, s, m);
}

template <int BITS, bool BF16, int AR, int MB>
void launch_fwd_m16_nb(const FwdMulti &m, int nb, hipStream_t s)
{
    constexpr int NST = m16_nst(BITS, MB, AR);
    switch (nb) {
    case 4:
        if constexpr (NST * m16_stage(BITS, 4, AR, MB) < M16_LDS) { launch_fwd_m16_one<BITS, BF16, 4, AR, MB>(m, s); return; }
        [[fallthrough]];
    case 3:
        if constexpr (NST * m16_stage(BITS, 3, AR, MB) < M16_LDS) { launch_fwd_m16_one<BITS, BF16, 3, AR, MB>(m, s); return; }
        [[fallthrough]];
    case 2:
        if constexpr (NST * m16_stage(BITS, 2, AR, MB) < M16_LDS) { launch_fwd_m16_one<BITS, BF16, 2, AR, MB>(m, s); return; }
        [[fallthrough]];
    default:
        if constexpr (NST * m16_stage(BITS, 1, AR, MB) < M16_LDS) launch_fwd_m16_one<BITS, BF16, 1, AR, MB>(m, s);
    }
}

// Serves the call if its shape allows: up to 32 token rows (above 16, or with more than 16 adapter rows: not for 3-bit
// codes), K and the group size
// multiples of 128 (a wave's columns of a stage then share their group constants), t either computed here from at most
// 32 adapter rows or handed in, and room in LDS for the stages of at least two 16-row blocks (one block would pull x
// through every compute unit once per 16 weight rows).
template <int BITS, bool BF16>
bool launch_fwd_m16(const FwdMulti &m, int rg, hipStream_t s)
{
    const FwdArgs &a = m.p[0];
    if (a.M > 32 || a.K % 128 != 0 || (a.K / a.ng) % 128 != 0 || rg > 2 || (rg == 0 && a.r > 64)) return false;
    const int mb = a.M > 16 ? 2 : 1;
    if (BITS == 3 && (mb == 2 || rg == 2)) return false;   // 64-column slices would cut the 12-byte units of 3-bit codes
    for (int i = 0; i < m.count; ++i) {
        const FwdArgs &b = m.p[i];            // 16-byte requests: aligned arrays, constants in whole pieces
        const uintptr_t bits_or = (uintptr_t)b.x | (uintptr_t)b.packed | (uintptr_t)b.scales | (uintptr_t)b.zeros |
                                  (uintptr_t)b.zpacked | (rg ? (uintptr_t)b.A : 0);
        if ((bits_or & 15) != 0 || ((long)b.N * b.ng) % 16 != 0 || ((long)b.N * m16_zrow(b)) % 16 != 0) return false;
    }
    const int ar = rg == 0 ? 0 : (a.r <= 8 ? 8 : (a.r <= 16 ? 16 : 32));
    const int nb_max = m16_nb_max<BITS>(ar, a.ng, m16_zrow(a), mb);
    if (nb_max < 2) return false;
    // one round of the 256 compute units if the rows allow it; siblings that do not fit one round together go one by one
    int nb = 0;
    for (int cand = 1; cand <= nb_max && nb == 0; ++cand) {
        int wgs = 0;
        for (int i = 0; i < m.count; ++i) wgs += (blocks16(m.p[i].N) + cand - 1) / cand;
        if (wgs <= 256) nb = cand;
    }
    if (nb == 0 && m.count > 1) {
        for (int i = 0; i < m.count; ++i) {
            FwdMulti one{};
            one.count = 1;
            one.p[0] = m.p[i];
            launch_fwd_m16<BITS, BF16>(one, rg, s);
        }
        return true;
    }
    if (nb == 0) nb = nb_max;
    if (mb == 1) {
        switch (ar) {
        case 0: launch_fwd_m16_nb<BITS, BF16, 0, 1>(m, nb, s); break;
        case 8: launch_fwd_m16_nb<BITS, BF16, 8, 1>(m, nb, s); break;
        case 16: launch_fwd_m16_nb<BITS, BF16, 16, 1>(m, nb, s); break;
        default:
            if constexpr (BITS != 3) launch_fwd_m16_nb<BITS, BF16, 32, 1>(m, nb, s);
        }
    } else if constexpr (BITS != 3) {
        switch (ar) {
        case 0: launch_fwd_m16_nb<BITS, BF16, 0, 2>(m, nb, s); break;
        case 8: launch_fwd_m16_nb<BITS, BF16, 8, 2>(m, nb, s); break;
        case 16: launch_fwd_m16_nb<BITS, BF16, 16, 2>(m, nb, s); break;
        default: launch_fwd_m16_nb<BITS, BF16, 32, 2>(m, nb, s); break;
        }
    }
    return true;
}

}  // namespace

}  // namespace qlora
