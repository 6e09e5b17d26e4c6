// Small token counts, backward pass (M <= 16; M <= 32 where the staged kernel applies): see gemv_fwd.hip for the regime.  Two launches: row-sliced partial
// dX = dY Wd with the 8-row in-register transposition of the packed codes (Sec. 3.1: transpose + unpack + matmul in
// one kernel) and partial u = dY B; then the slice sums, sc u A, dA = sc u^T x and dB = sc dY^T t.
#include "gemv_common.hpp"

namespace qlora {

namespace {

// ------------------------------------------------------------------------------------------------ backward
// Workgroup (cb, sp): weight columns [CB cb, +CB), CB = 16 * CL, rows n of slice sp; wave w takes 32-row chunks
// w, w+4, ...  Lane (wc = lane % 16, q = lane / 16) holds the CL codes of columns CB cb + CL wc .. of rows
// chunk + 8 q + e, e = 0..7.  MFMA number c of a chunk multiplies dY[m, 32 rows] with the codes at column
// CL wc + c of those rows: D_c[m][k = CB cb + CL wc + c].
template <int BITS>
struct BwdShape {
    static constexpr int CL = BITS == 3 ? 32 : (BITS == 2 ? 16 : 8);   // columns per lane: one packed word (3-bit: three)
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
    float *upartial;      // [slices][16][64] ([slices][32][64] above 16 token rows)
    int M, N, K, r, ng, rows_per_slice;
    uint32_t magic;
    const uint32_t *zpacked;   // zero-points in their bit-packed storage form [N, zw] (then `zeros` is not read), or NULL
    int zw;                    // words per row of zpacked
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

// ------------------------------------------------------------------------------- backward, staged through LDS
// The same products as gemv_bwd_body, with every operand brought in by direct-to-LDS loads instead of fragment-wise
// loads: a 32-row chunk costs the kernel above eight 4-byte loads of packed words plus up to sixteen 1- and 2-byte
// loads of group constants per lane, and what bounds it is the number of such instructions, not the bytes.  Here a
// workgroup of eight waves walks its row slice in stages of 256 rows, NST stages in flight; a stage is the rows'
// packed words inside the column block (RB bytes per row), the 16 x 256 piece of dY and, per row, the 16-byte piece of
// the scale table and the one of the zero-point table that hold the block's one or two groups (such a pair never
// straddles two pieces: with two groups per block the number of groups per row is even).  Wave w multiplies chunk w
// of every stage.  One step ahead of their use the windows are turned into per-group arrays of fp16 scales and -z
// over the rows, so that a lane picks up the constants of its eight rows with two 16-byte reads.
//
// LDS rows of a stage are permuted (bits 0-2 and 3-4 of the row index change places): the four rows 8 q + e that a
// wave reads together then lie in four different bank ranges.  The dY pieces are permuted by the token row.
constexpr int BS_RS = 256, BS_NW = 8;

// MB: 16-row token blocks (1, or 2 for 17 to 32 token rows: a stage then holds 32 rows of dY, three stages fit, and
// 8-bit codes, whose rows are twice as wide, do not)
template <int BITS, int MB = 1>
struct BwdStaged {
    using S = BwdShape<BITS>;
    static constexpr int RB = S::CB * BITS / 8;             // bytes of a weight row inside the column block
    static constexpr int PPR = RB / 16;
    static constexpr int WBYTES = BS_RS * RB, DYB = 16 * MB * BS_RS * 2, SZB = BS_RS * 32;
    static constexpr int STAGE = WBYTES + DYB + SZB;
    static constexpr int NST = BITS == 8 || MB == 2 ? 3 : 4;
    static constexpr int WD = WBYTES / 1024 / BS_NW;        // weight requests per wave and stage
    static constexpr int WIN = 1;                           // window requests per wave and stage
    static constexpr int GRP = WD + WIN + MB;               // ... and all requests: windows, MB of dY, WD
    static constexpr int CONV = 2 * 2 * 2 * BS_RS * 2;      // [parity][scale | -z][group][row] fp16
    static constexpr int RED = BS_NW * 16 * S::CB * 4;      // the waves' partial sums of one token block
    static constexpr int LDS = NST * STAGE + CONV > RED ? NST * STAGE + CONV : RED;
    static constexpr bool FITS = LDS <= 160 * 1024;
    static_assert(BITS != 3 && WBYTES % (1024 * BS_NW) == 0 && (FITS || MB == 2), "stage shape");
};

__device__ __forceinline__ int bs_perm(int row) { return (row & ~31) | ((row & 7) << 2) | ((row >> 3) & 3); }
__device__ __forceinline__ int bs_unperm(int p) { return (p & ~31) | ((p & 3) << 3) | ((p >> 2) & 7); }

template <int N>
__device__ __forceinline__ void bs_wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int BITS, bool BF16, int MB>
__device__ __forceinline__ void gemv_bwd_staged_body(const BwdArgs &a, const int cb, const int sp_local, const int sp)
{
    using S = BwdShape<BITS>;
    using T = BwdStaged<BITS, MB>;
    constexpr int CL = S::CL, WORDS = S::WORDS, CB = S::CB, NW = BS_NW, NT = NW * 64;
    constexpr int RB = T::RB, PPR = T::PPR, NST = T::NST, WD = T::WD, GRP = T::GRP, STAGE = T::STAGE;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wc = lane & 15, q = lane >> 4;
    const int N = a.N, K = a.K, ng = a.ng;
    const int Kw = K * BITS / 32;
    const int nbeg = sp_local * a.rows_per_slice, nend = min(N, nbeg + a.rows_per_slice);
    const int rows = nend - nbeg, stages = (rows + BS_RS - 1) / BS_RS;
    if (rows <= 0) {                                                        // a slice past the last row (uniform): zeros
        for (int e = threadIdx.x; e < a.M * CB; e += NT) a.partial[((long)sp * a.M + e / CB) * K + cb * CB + e % CB] = 0.f;
        return;
    }
    const int g0 = group_of(cb * CB, a.magic);                              // first group of the column block
    const int gl = group_of(cb * CB + CL * wc, a.magic) - g0;              // this lane's columns: 0 or 1
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lds;
    uint16_t *conv = (uint16_t *)(lds + NST * STAGE);                       // [parity][scale | -z][group][BS_RS]

    // ---- this lane's part of the requests of a stage
    const uint32_t *wbase = a.packed + (long)nbeg * Kw + cb * (RB / 4);
    const uint32_t row_bytes = (uint32_t)Kw * 4u;
    const int row_max = N - 1 - nbeg;                                       // rows past the matrix repeat its last row
    int w_row[WD];
    uint32_t w_pc[WD];
#pragma unroll
    for (int c = 0; c < WD; ++c) {
        const int e = 64 * (wave + NW * c) + lane;
        w_row[c] = bs_unperm(e / PPR);
        w_pc[c] = (uint32_t)(e % PPR) * 16u;
    }
    // dY: request `wave` of token block b moves token rows 16 b + 2 wave, + 1; slot s of a row holds piece s ^ (row % 16)
    const int dy_m = 2 * wave + (lane >> 5), dy_piece = (lane & 31) ^ dy_m;
    uint32_t dy_row[MB];
#pragma unroll
    for (int b = 0; b < MB; ++b) dy_row[b] = (uint32_t)min(16 * b + dy_m, a.M - 1) * (uint32_t)N * 2u;
    // windows: request `wave` moves rows 32 wave .. 32 wave + 32, lane l the scale piece (l even) or the zero-point
    // piece (l odd) of row 32 wave + l / 2
    // (bit-packed zero-points: the piece of the row's words that holds the block's groups; two groups of a block
    // share a word, the code widths here being powers of two)
    const bool zpk = a.zpacked != nullptr;                                  // workgroup-uniform
    const uint32_t zrow = zpk ? (uint32_t)a.zw * 4u : (uint32_t)ng, zg0 = zpk ? ((uint32_t)(g0 * BITS) >> 5) * 4u : (uint32_t)g0;
    const uint8_t *zsrc = zpk ? (const uint8_t *)a.zpacked : a.zeros;
    const uint32_t s_all = (uint32_t)N * ng * 2u, z_all = (uint32_t)N * zrow;
    auto issue = [&](int st) {
        const uint32_t base = lds0 + (uint32_t)(st % NST) * STAGE;
        {
            const int row = 32 * wave + (lane >> 1);
            const uint32_t n = (uint32_t)min(st * BS_RS + row, row_max) + nbeg;
            const uint32_t e = n * ng + g0;
            const uint32_t sat = (e * 2u) & ~15u, zat = (n * zrow + zg0) & ~15u;
            const uint8_t *src = (lane & 1) == 0 ? (const uint8_t *)a.scales + (sat + 16u <= s_all ? sat : 0u)
                                                 : zsrc + (zat + 16u <= z_all ? zat : 0u);
            dma16_at(src, base + T::WBYTES + T::DYB + (uint32_t)wave * 1024u);
        }
#pragma unroll
        for (int b = 0; b < MB; ++b) {
            const int n = nbeg + st * BS_RS + 8 * dy_piece;                 // N % 8 == 0: a piece is inside or outside
            dma16(a.dy, dy_row[b] + (n < N ? (uint32_t)n * 2u : 0u),
                  base + T::WBYTES + (uint32_t)(8 * b + wave) * 1024u);
        }
#pragma unroll
        for (int c = 0; c < WD; ++c)
            dma16(wbase, (uint32_t)min(st * BS_RS + w_row[c], row_max) * row_bytes + w_pc[c],
                  base + (uint32_t)(wave + NW * c) * 1024u);
    };
    // the windows of stage st become scales and -z per group and row (thread = row); rows past the slice get scale 0
    auto convert = [&](int st) {
        if (threadIdx.x < BS_RS) {
            const int row = threadIdx.x, rs = st * BS_RS + row;
            const uint8_t *win = lds + (size_t)(st % NST) * STAGE + T::WBYTES + T::DYB + row * 32;
            const uint32_t n = (uint32_t)min(rs, row_max) + nbeg, e = n * ng + g0;
            const uint32_t sw = *(const uint32_t *)(win + ((e * 2u) & 12u)) >> (8 * ((e * 2u) & 3u));     // two scales
            const uint32_t za = n * zrow + zg0;                                                          // as in issue()
            uint32_t zw = *(const uint32_t *)(win + 16 + (za & 12u));                                    // two zero-points
            zw >>= zpk ? (uint32_t)(g0 * BITS) & 31u : 8u * (za & 3u);
            const uint32_t zbits = zpk ? (uint32_t)BITS : 8u, zmask = (1u << zbits) - 1u;
            uint16_t *dst = conv + (st & 1) * (4 * BS_RS) + row;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                dst[g * BS_RS] = rs < rows ? (uint16_t)(sw >> (16 * g)) : (uint16_t)0;
                dst[(2 + g) * BS_RS] = f32_to_f16_bits(-(float)((zw >> (zbits * g)) & zmask));
            }
        }
    };

    float4_t acc[MB][CL];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int c = 0; c < CL; ++c) acc[b][c] = float4_t{0.f, 0.f, 0.f, 0.f};

    // Requests complete in the order they were made, so "stage st has landed" is a bound on the number of requests
    // still outstanding: those of the stages requested after it.  wait_later(n, keep): at most n later stages and, of
    // the stage next in line, everything but its first `keep` requests (the windows) may be outstanding.
    auto wait_later = [&](int later, int keep) {      // workgroup-uniform arguments
        if (later >= 3) bs_wait_vm<3 * GRP>();        // (only without keep: the start-up)
        else if (later == 2) { if (keep) bs_wait_vm<2 * GRP - T::WIN>(); else bs_wait_vm<2 * GRP>(); }
        else if (later == 1) { if (keep) bs_wait_vm<GRP - T::WIN>(); else bs_wait_vm<GRP>(); }
        else bs_wait_vm<0>();
    };
    static_assert(NST <= 4, "wait_later covers three stages in flight");
    const int ahead = min(NST - 1, stages);            // stages requested before the first is used
    for (int st = 0; st < ahead; ++st) issue(st);
    // the windows of stage 0 (its first request) have landed
    if (ahead == 3) bs_wait_vm<3 * GRP - T::WIN>();
    else if (ahead == 2) bs_wait_vm<2 * GRP - T::WIN>();
    else bs_wait_vm<GRP - T::WIN>();
    __syncthreads();
    convert(0);
    for (int st = 0; st < stages; ++st) {
        // stage st and the windows of stage st + 1
        const int later = min(NST - 2, stages - 1 - st);
        wait_later(later, later > 0);
        __syncthreads();                              // ... for every wave; the arrays written by convert are visible
        if (st + NST - 1 < stages) issue(st + NST - 1);   // into the buffer every wave has left with the step before
        if (st + 1 < stages) convert(st + 1);
        const uint8_t *buf = lds + (size_t)(st % NST) * STAGE;
        const int rs0 = st * BS_RS + 32 * wave + 8 * q;                    // first of this lane's eight rows
        if (st * BS_RS + 32 * wave >= rows) continue;                      // wave-uniform: the chunk is past the slice
        const bool in = rs0 < rows;                                        // slices end on multiples of 8
        uint32_t w[8][WORDS];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint8_t *src = buf + (32 * wave + 4 * e + q) * RB + wc * (WORDS * 4);
            if constexpr (WORDS == 2) {
                const u32x2_t v = *(const u32x2_t *)src;
                w[e][0] = v[0];
                w[e][1] = v[1];
            } else {
                w[e][0] = *(const uint32_t *)src;
            }
        }
        u16x8_t df[MB];
#pragma unroll
        for (int b = 0; b < MB; ++b) {
            df[b] = *(const u16x8_t *)(buf + T::WBYTES + (16 * b + wc) * 512 + (((4 * wave + q) ^ wc) * 16));
            if (!in) df[b] = ZERO8;
        }
        const uint16_t *cs = conv + (st & 1) * (4 * BS_RS) + gl * BS_RS + 32 * wave + 8 * q;
        // read with the element type they were written with, then regrouped into pairs
        const u32x4_t sv = __builtin_bit_cast(u32x4_t, *(const u16x8_t *)cs);
        const u32x4_t zv = __builtin_bit_cast(u32x4_t, *(const u16x8_t *)(cs + 2 * BS_RS));
        if constexpr (BF16) {
            float s[8], z[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                s[e] = f16_bits_to_f32((uint16_t)(sv[e >> 1] >> (16 * (e & 1))));
                z[e] = -f16_bits_to_f32((uint16_t)(zv[e >> 1] >> (16 * (e & 1))));
            }
#pragma unroll
            for (int c = 0; c < CL; ++c) {
                u16x8_t wf;
#pragma unroll
                for (int e = 0; e < 8; ++e) wf[e] = to16<BF16>(((float)code_of<BITS, WORDS>(w[e], c) - z[e]) * s[e]);
#pragma unroll
                for (int b = 0; b < MB; ++b) acc[b][c] = mfma16<BF16>(df[b], wf, acc[b][c]);   // D[m = 4q+v][column CL wc + c]
            }
        } else {
            half2_t s2[4], nz2[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t sw = sv[i], zw = zv[i];       // (a bit cast straight from a vector element reads element 0)
                s2[i] = __builtin_bit_cast(half2_t, sw);
                nz2[i] = __builtin_bit_cast(half2_t, zw);
            }
#pragma unroll
            for (int c = 0; c < CL; ++c) {
                const u16x8_t wf = dequant_rows8_f16<BITS, WORDS>(w, c, s2, nz2);
#pragma unroll
                for (int b = 0; b < MB; ++b) acc[b][c] = mfma16<BF16>(df[b], wf, acc[b][c]);
            }
        }
    }
    __syncthreads();                                  // every request has landed (the last wait was for all)
    // ---- the waves' sums meet in LDS: [wave][m][CB] floats, then every thread adds up four columns of one row.  A
    //      lane's CL columns are P = CL / 4 pieces of 16 bytes; piece j sits in slot j ^ f(lane) of the lane's P, with f
    //      chosen so that the sixteen lanes of one store fall on sixteen different bank groups.
    //      (one token block at a time: the area holds the sums of sixteen token rows)
    constexpr int P = CL / 4;
    float *red = (float *)lds;
    const int f = (wc / (16 / P)) & (P - 1);
#pragma unroll
    for (int b = 0; b < MB; ++b) {
        if (b > 0) __syncthreads();                   // the sums of the block before have been read
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float *dst = red + ((size_t)wave * 16 + 4 * q + v) * CB + CL * wc;
#pragma unroll
            for (int j = 0; j < P; ++j)
                *(float4_t *)(dst + 4 * (j ^ f)) =
                    float4_t{acc[b][4 * j][v], acc[b][4 * j + 1][v], acc[b][4 * j + 2][v], acc[b][4 * j + 3][v]};
        }
        __syncthreads();
        for (int e = threadIdx.x; e < 16 * CB / 4; e += NT) {
            const int m = 16 * b + e / (CB / 4), k4 = e % (CB / 4);
            if (m >= a.M) continue;
            const int lw = k4 / P, slot = P * lw + ((k4 % P) ^ ((lw / (16 / P)) & (P - 1)));
            float4_t v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < NW; ++w) v += *(const float4_t *)(red + ((size_t)w * 16 + (m & 15)) * CB + 4 * slot);
            *(float4_t *)(a.partial + ((long)sp * a.M + m) * K + cb * CB + 4 * k4) = v;
        }
    }
}

// u = dY B of one row slice (the workgroup past the last column block of every slice): B^T fragments gathered
// column-wise, four 32-row chunks in flight per wave
template <bool BF16, int MB>
__device__ __forceinline__ void gemv_bwd_u_body(const BwdArgs &a, const int sp_local, const int sp)
{
    constexpr int NW = BS_NW, NT = NW * 64, XR = 16 * MB;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    float (*ured)[XR][64 + 1] = (float (*)[XR][64 + 1])lds;                 // [NW][XR][65], 33 KB per token block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wc = lane & 15, q = lane >> 4;
    const int N = a.N, r = a.r;
    const int nbeg = sp_local * a.rows_per_slice, nend = min(N, nbeg + a.rows_per_slice);
    float4_t uacc[MB][4];
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) uacc[b][gg] = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int nb = nbeg + wave * 32; nb < nend; nb += 32 * NW) {
        const int nn = nb + 8 * q;
        const bool in = nn < nend;                                          // slices end on multiples of 8
        u16x8_t df[MB];
#pragma unroll
        for (int b = 0; b < MB; ++b)
            df[b] = in ? *(const u16x8_t *)(a.dy + (long)min(16 * b + wc, a.M - 1) * N + nn) : ZERO8;
#pragma unroll
        for (int gg = 0; gg < 4; ++gg) {
            const int j = gg * 16 + wc;
            if (gg * 16 >= r) continue;                                     // uniform
            u16x8_t bf = ZERO8;
            if (in && j < r) {
#pragma unroll
                for (int e = 0; e < 8; ++e) bf[e] = a.B[(long)(nn + e) * r + j];
            }
#pragma unroll
            for (int b = 0; b < MB; ++b) uacc[b][gg] = mfma16<BF16>(df[b], bf, uacc[b][gg]);   // D[m = 4q+v][j = 16 gg + wc]
        }
    }
#pragma unroll
    for (int b = 0; b < MB; ++b)
#pragma unroll
        for (int gg = 0; gg < 4; ++gg)
#pragma unroll
            for (int v = 0; v < 4; ++v) ured[wave][16 * b + 4 * q + v][16 * gg + wc] = uacc[b][gg][v];
    __syncthreads();
    for (int e = threadIdx.x; e < XR * 64; e += NT) {         // a slice's u: XR rows of 64 columns
        const int m = e >> 6, j = e & 63;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) v += ured[w][m][j];
        a.upartial[(long)sp * (XR * 64) + e] = v;
    }
}

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

// grid (column blocks + 1, slices): the last workgroup of a slice computes u.  Workgroups are dealt to the eight XCDs
// round-robin by their linear index, and two neighbouring column blocks share the 128-byte lines of the packed rows
// (a block covers 64 bytes of a row at 2 and 4 bits): the work items are renumbered so that each XCD gets a
// contiguous run of (slice, column block) pairs, column block fastest, and a line is fetched into one L2 only.
template <int BITS, bool BF16, int MB>
__global__ __launch_bounds__(BS_NW * 64) void gemv_bwd_staged_kernel(const BwdMulti ma)
{
    const int gx = (int)gridDim.x, total = gx * (int)gridDim.y;
    const int linear = (int)blockIdx.y * gx + (int)blockIdx.x, die = linear & 7;
    const int item = die * (total >> 3) + min(die, total & 7) + (linear >> 3);
    const int sp = item / gx, cbx = item % gx;
    int pi = 0;
    while (pi + 1 < ma.count && sp >= ma.slice_end[pi]) ++pi;      // wave-uniform
    const BwdArgs a = ma.p[pi];
    const int sp_local = sp - (pi ? ma.slice_end[pi - 1] : 0);
    if (cbx + 1 == gx) {
        if (a.r > 0) gemv_bwd_u_body<BF16, MB>(a, sp_local, sp);
    } else {
        gemv_bwd_staged_body<BITS, BF16, MB>(a, cbx, sp_local, sp);
    }
}

// Second backward kernel (M <= 32), one thread per output element:
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
    float sc, beta;      // dA = beta * dA + ..., dB likewise (beta == 0: they are not read)
    const uint8_t *keep; // LoRA dropout: keep bits of x as bytes [M, K/8], or NULL
    float keep_scale;
    int r0;              // stacked adapters: adapter columns below r0 are frozen; dA is [r - r0, K], dB [N, r - r0]
    int ustride;         // floats of a slice's partial u: 64 columns x 16 or 32 token rows
};

// MASKED (a.keep != NULL) is a template argument: a test of the pointer inside the token loop kept the compiler from
// requesting the loop's loads together (4.5 -> 6.4 us per call).
template <bool BF16, bool MASKED>
__global__ __launch_bounds__(256) void gemv_bwd_finish_kernel(const FinishArgs a)
{
    __shared__ float side[32][64 + 1];       // u (dX and dA blocks) or t (dB blocks), as the 16-bit values they round to
    const int M = a.M, r = a.r, K = a.K, N = a.N;
    const int b = blockIdx.x;
    // The kernel is a few dependent memory round trips long, so every load that can be is requested before the first
    // result is needed: a dX thread asks for its slice sums (sixteen at a time) before the block turns to u.
    const long idx_x = (long)b * 256 + threadIdx.x;
    const bool x_thread = b < a.xb && idx_x < (long)M * K;
    const long stride = (long)M * K;
    float pv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pv[i] = x_thread && i < a.slices ? a.partial[i * stride + idx_x] : 0.f;
    if (b < a.xb + a.ab) {
        for (int e = threadIdx.x; e < M * r; e += 256) {
            const int m = e / r, j = e % r;
            const float *up = a.upartial + m * 64 + j;
            float v = 0.f;
            for (int s0 = 0; s0 < a.slices; s0 += 16) {      // sixteen slices requested together, summed in slice order
                float uv[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) uv[i] = s0 + i < a.slices ? up[(long)(s0 + i) * a.ustride] : 0.f;
#pragma unroll
                for (int i = 0; i < 16; ++i) v += uv[i];
            }
            side[m][j] = cvt16<BF16>(to16<BF16>(v));
        }
    } else {
        for (int e = threadIdx.x; e < M * r; e += 256) side[e / r][e % r] = cvt16<BF16>(a.t[e]);
    }
    __syncthreads();
    if (b < a.xb) {
        if (!x_thread) return;
        const long idx = idx_x;
        const int m = (int)(idx / K), k = (int)(idx % K);
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) v += pv[i];                 // slice order; the entries past the last slice are zero
        for (int s0 = 16; s0 < a.slices; s0 += 16) {
            float more[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) more[i] = s0 + i < a.slices ? a.partial[(s0 + i) * stride + idx] : 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) v += more[i];
        }
        float lo = 0.f;
        for (int j = 0; j < r; ++j) lo += side[m][j] * cvt16<BF16>(a.A[(long)j * K + k]);
        if constexpr (MASKED) lo = ((a.keep[(long)m * (K / 8) + (k >> 3)] >> (k & 7)) & 1) ? lo * a.keep_scale : 0.f;
        a.dx[idx] = to16<BF16>(v + a.sc * lo);
    } else if (b < a.xb + a.ab) {
        const long idx = (long)(b - a.xb) * 256 + threadIdx.x;
        if (idx >= (long)(r - a.r0) * K) return;
        const int j = a.r0 + (int)(idx / K), k = (int)(idx % K);
        float v = 0.f;
        for (int m = 0; m < M; ++m) {
            float xv = cvt16<BF16>(a.x[(long)m * K + k]);
            if constexpr (MASKED) xv = ((a.keep[(long)m * (K / 8) + (k >> 3)] >> (k & 7)) & 1) ? xv * a.keep_scale : 0.f;
            v += side[m][j] * xv;
        }
        a.dA[idx] = a.beta == 0.f ? a.sc * v : fmaf(a.beta, a.dA[idx], a.sc * v);
    } else {
        const long idx = (long)(b - a.xb - a.ab) * 256 + threadIdx.x;
        if (idx >= (long)(r - a.r0) * N) return;
        const int j = a.r0 + (int)(idx / N), n = (int)(idx % N);
        float v = 0.f;
        for (int m = 0; m < M; ++m) v += cvt16<BF16>(a.dy[(long)m * N + n]) * side[m][j];
        float *dst = a.dB + (long)n * (r - a.r0) + (j - a.r0);
        *dst = a.beta == 0.f ? a.sc * v : fmaf(a.beta, *dst, a.sc * v);
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
    float sc, beta;
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
            for (int s0 = sb; s0 < se; s0 += 16) {
                float uv[16];
#pragma unroll
                for (int i16 = 0; i16 < 16; ++i16) uv[i16] = s0 + i16 < se ? up[(long)(s0 + i16) * 1024] : 0.f;
#pragma unroll
                for (int i16 = 0; i16 < 16; ++i16) v += uv[i16];
            }
            side[slot][m][j] = cvt16<BF16>(to16<BF16>(v));
        }
    };
    if (b < a.xb) {
        // the thread's slice sums are requested (sixteen at a time) before the block turns to u
        const long idx = (long)b * 256 + threadIdx.x, stride = (long)M * K;
        const bool live = idx < stride;
        float pv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) pv[i] = live && i < a.slices ? a.partial[i * stride + idx] : 0.f;
        for (int i = 0; i < a.count; ++i) sum_u(i, i);
        __syncthreads();
        if (!live) return;
        const int m = (int)(idx / K), k = (int)(idx % K);
        float v = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) v += pv[i];                 // slice order; the entries past the last slice are zero
        for (int s0 = 16; s0 < a.slices; s0 += 16) {
            float more[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) more[i] = s0 + i < a.slices ? a.partial[(s0 + i) * stride + idx] : 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) v += more[i];
        }
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
        a.p[i].dA[idx] = a.beta == 0.f ? a.sc * v : fmaf(a.beta, a.p[i].dA[idx], a.sc * v);
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
        float *dst = pr.dB + (long)n * r + j;
        *dst = a.beta == 0.f ? a.sc * v : fmaf(a.beta, *dst, a.sc * v);
    }
}

// whether the staged kernel takes the launch: column blocks that divide K and hold at most two groups, 16-byte
// aligned operands and tables of whole 16-byte pieces (they are fetched by direct-to-LDS loads), packed rows
// addressed with 32 bits
template <int BITS>
bool bwd_staged_applies(const BwdMulti &m)
{
    if constexpr (BITS == 3) {
        return false;
    } else {
        if (m.p[0].M > 16 && (m.count > 1 || !BwdStaged<BITS, 2>::FITS)) return false;
        constexpr int CB = BwdShape<BITS>::CB;
        for (int i = 0; i < m.count; ++i) {
            const BwdArgs &a = m.p[i];
            const int G = a.K / a.ng;
            if (a.K % CB != 0 || !(G % CB == 0 || (CB % G == 0 && CB / G <= 2))) return false;
            if ((long)a.N * a.K * BITS / 8 >= (1ll << 32) || ((long)a.N * a.ng) % 16 != 0) return false;   // whole 16-byte pieces of constants
            const uintptr_t bits_or = (uintptr_t)a.dy | (uintptr_t)a.packed | (uintptr_t)a.scales | (uintptr_t)a.zeros |
                                      (uintptr_t)a.zpacked;
            if ((bits_or & 15) != 0 || (a.zpacked && ((long)a.N * a.zw) % 4 != 0)) return false;
        }
        return true;
    }
}

// *taken = false and nothing launched: bit-packed zero-points or more than 16 token rows were handed in and the staged
// kernel, the one that takes them, does not take the shape
template <int BITS, bool BF16>
void launch_bwd_bits(const BwdMulti &m, hipStream_t s, bool *taken)
{
    *taken = true;
    if constexpr (BITS != 3) {
        if (bwd_staged_applies<BITS>(m)) {
            const dim3 grid(m.p[0].K / BwdShape<BITS>::CB + 1, m.slice_end[m.count - 1]);
            if (m.p[0].M <= 16) {
                auto kern = gemv_bwd_staged_kernel<BITS, BF16, 1>;
                ensure_dynamic_lds((const void *)kern, BwdStaged<BITS>::LDS);
                QLORA_LAUNCH(kern, grid, dim3(BS_NW * 64), BwdStaged<BITS>::LDS, s, m);
            } else if constexpr (BwdStaged<BITS, 2>::FITS) {
                auto kern = gemv_bwd_staged_kernel<BITS, BF16, 2>;
                constexpr int lds2 = BwdStaged<BITS, 2>::LDS;
                ensure_dynamic_lds((const void *)kern, lds2);
                QLORA_LAUNCH(kern, grid, dim3(BS_NW * 64), lds2, s, m);
            }
            return;
        }
    }
    if (m.p[0].zpacked || m.p[0].M > 16) {      // the kernels below read unpacked zero-points and hold 16 token rows
        *taken = false;
        return;
    }
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
                QLORA_LAUNCH((gemv_bwd_kernel<BITS, BF16, 8, 2>), grid, dim3(512), 0, s, m.p[0]);
                return;
            }
        }
        QLORA_LAUNCH((gemv_bwd_kernel<BITS, BF16, 4, 2>), grid, dim3(256), 0, s, m.p[0]);
        return;
    }
    if constexpr (BITS != 3) {
        if (eight) {
            QLORA_LAUNCH((gemv_bwd_siblings_kernel<BITS, BF16, 8, 2>), grid, dim3(512), 0, s, m);
            return;
        }
    }
    QLORA_LAUNCH((gemv_bwd_siblings_kernel<BITS, BF16, 4, 2>), grid, dim3(256), 0, s, m);
}

int bwd_cb(int bits) { return bits == 3 ? BwdShape<3>::CB : (bits == 2 ? BwdShape<2>::CB : (bits == 4 ? BwdShape<4>::CB : BwdShape<8>::CB)); }

}  // namespace

int gemv_bwd_slices(int N, int K, int bits)
{
    const int colblocks = (K + bwd_cb(bits) - 1) / bwd_cb(bits) + 1;     // + 1: the workgroup that computes u
    int slices = 256 / colblocks;                        // one workgroup per compute unit, in one round: every extra
    if (slices < 1) slices = 1;                          // slice costs another M x K block of partial sums
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
    const int colblocks = (K + bwd_cb(bits) - 1) / bwd_cb(bits) + 1;
    const int target = 256 / colblocks < 1 ? 1 : 256 / colblocks;
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

bool launch_bwd_small(const Problem &p, int count, const void *const *dy, const void *x,
                      const uint32_t *const *packed, const void *const *scales, const uint8_t *const *zeros,
                      const void *const *A, const void *const *B, const void *const *t, void *dx, float *const *dA,
                      float *const *dB, const int *N, float *partial, float *upartial, float beta, const uint32_t *keep,
                      float keep_scale, int frozen, hipStream_t s, const uint32_t *const *zpacked)
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
                         rows_per_slice, group_magic(p.G), zpacked ? zpacked[i] : nullptr,
                         zpacked ? zero_words(p.K / p.G, p.bits) : 0};
        end += slices[i];
        m.slice_end[i] = end;
    }
    bool taken = true;
    QLORA_BITS_DTYPE(launch_bwd_bits, m, s, &taken);
    if (!taken) return false;
    const int rt = count == 1 ? p.r - frozen : p.r;     // adapter columns with gradients (siblings: no frozen part)
    const int xb = (int)(((long)p.M * p.K + 255) / 256), ab = (int)(((long)rt * p.K + 255) / 256);
    if (count == 1) {
        const int bb = (int)(((long)rt * N[0] + 255) / 256);
        const FinishArgs f{partial, upartial, (const uint16_t *)(A ? A[0] : nullptr), (const uint16_t *)x,
                           (const uint16_t *)dy[0], (const uint16_t *)(t ? t[0] : nullptr), (uint16_t *)dx,
                           dA ? dA[0] : nullptr, dB ? dB[0] : nullptr, p.M, N[0], p.K, p.r, total, xb, ab, p.sc, beta,
                           (const uint8_t *)keep, keep_scale, frozen, p.M > 16 ? 2048 : 1024};
        const dim3 grid(xb + ab + bb), block(256);
        if (keep) {
            if (p.bf16) QLORA_LAUNCH((gemv_bwd_finish_kernel<true, true>), grid, block, 0, s, f);
            else QLORA_LAUNCH((gemv_bwd_finish_kernel<false, true>), grid, block, 0, s, f);
        } else {
            if (p.bf16) QLORA_LAUNCH((gemv_bwd_finish_kernel<true, false>), grid, block, 0, s, f);
            else QLORA_LAUNCH((gemv_bwd_finish_kernel<false, false>), grid, block, 0, s, f);
        }
        return true;
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
    f.beta = beta;
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
        QLORA_LAUNCH((gemv_bwd_finish_siblings_kernel<true>), dim3(blocks), dim3(256), 0, s, f);
    else
        QLORA_LAUNCH((gemv_bwd_finish_siblings_kernel<false>), dim3(blocks), dim3(256), 0, s, f);
    return true;
}

}  // namespace qlora
