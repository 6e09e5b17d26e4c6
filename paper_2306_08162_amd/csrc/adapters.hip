// Rank-r side of the layer (Fig. 1, green LoRA branch): t = x A^T, u = dY B and the gradients of the only
// trainable parameters, dA and dB (Sec. 3.1).  All four are skinny contractions that read x or dY once, so they
// are HBM-bound; they run on v_mfma_f32_16x16x32 so that their cost does not grow with the rank, accumulate in
// fp32 and reduce in a fixed order (no float atomics): results are bitwise reproducible.
#include "common.hpp"
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

// LoRA dropout (Appendix B trains with a rate of 0.05; it acts on the input of the low-rank branch only): the keep
// mask is one bit per element of x, bit k % 32 of word k / 32 of the row, i.e. one byte per 8-element fragment.
__device__ __forceinline__ u16x8_t keep_halves(u16x8_t v, uint32_t keep_byte)
{
    u32x4_t w = __builtin_bit_cast(u32x4_t, v);
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint32_t lo = (keep_byte >> (2 * d)) & 1u, hi = (keep_byte >> (2 * d + 1)) & 1u;
        w[d] &= lo * 0xFFFFu + hi * 0xFFFF0000u;
    }
    return __builtin_bit_cast(u16x8_t, w);
}

// ------------------------------------------------------------------------------------------------------------
// out[M,r] = act[M,C] * small[r,C]^T        (t = x A^T with small = A;  u = dY B with small = B^T)
//
// A workgroup of 8 waves owns 8 or 16 token rows (SK_ROWS: the MFMA block has 16; with 8 the upper half of the block
// stays zero and there are twice as many workgroups, which pays while 16-row workgroups would not fill the chip:
// 1.2 us per launch at 2048 x 4096).  Byte offsets of the loads are 32-bit: the entry points accept at most 2^31
// elements per activation matrix.
// ------------------------------------------------------------------------------------------------------------
constexpr int SK_WAVES = 8;

// Both operands are staged through LDS: every wave walks
// 64-column stretches of the contraction (wave w the stretches w, w + 8, ...) and pulls the stretch of its token rows
// and of `small` into one of two private LDS buffers with direct-to-LDS loads, the next stretch in flight while this
// one is multiplied; no workgroup barrier in the loop.  (Fragment loads straight from global memory are 16 bytes out
// of each of 16 rows per instruction: at rank 32 that kernel took 12.9 us at 2048 x 4096, this one 7.3; at rank 8
// 6.9 against 6.0.)
//   token rows: 8 rows x 128 bytes per load, the 16-byte pieces of a row XOR-swizzled by the row number so that
//               the fragment reads of 16 rows collide at most pairwise;
//   NATURAL = false (t = x A^T): `small` is [r, C], its rows are staged like token rows;
//   NATURAL = true  (u = dY B):  `small` is [C, r], the contraction index is the strided one; the stretch's 64 rows
//               are one contiguous block, copied as it lies, and the MFMA operand is gathered with the transposing
//               LDS read (in a block of 16 lanes, lane 4e+g supplies the address of four columns of one row; lane i
//               receives column i%4 of the rows supplied by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4).
constexpr int SS_COLS = 64;
//   MASKED (t under LoRA dropout, out = keep_scale * (x * keep) A^T): the keep bits of the stretch, 8 bytes per token
//               row, come in with one 4-byte-per-lane load and are applied to the fragments as they are read.
template <int RG, int SK_ROWS, bool NATURAL, bool MASKED>
constexpr int ss_buf_bytes()      // operands of one stretch (+ 256 bytes for keep bits)
{
    return (NATURAL ? SK_ROWS * 128 + SS_COLS * RG * 16 * 2 : (SK_ROWS + 16 * RG) * 128) + (MASKED ? 256 : 0);
}
template <bool BF16, int RG, int SK_ROWS, bool NATURAL, bool MASKED>
__global__ __launch_bounds__(SK_WAVES * 64) void skinny_rows_staged_kernel(const uint16_t *__restrict__ act,
                                                                          const uint16_t *__restrict__ small,
                                                                          uint16_t *__restrict__ out, int M, int C, int r,
                                                                          const uint8_t *__restrict__ keep, float keep_scale)
{
    static_assert(!(NATURAL && MASKED), "the mask belongs to x, the activation operand of t = x A^T");
    extern __shared__ __attribute__((aligned(16))) char ss_lds[];   // [SK_WAVES][2] buffers; then the final sum
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4_t *lds4_t;
    constexpr int BUF = ss_buf_bytes<RG, SK_ROWS, NATURAL, MASKED>(), MASK_OFF = BUF - 256;
    constexpr int XDMA = SK_ROWS / 8;                // loads of token rows per stretch
    constexpr int SDMA_MAX = 2 * RG;                 // loads of `small` per stretch, at most (16 RG rows or 64 x 16 RG columns)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int m0 = blockIdx.x * SK_ROWS;
    const int li = lane & 15, q = lane >> 4;
    const bool rowin = li < SK_ROWS;
    char *mine = ss_lds + wave * (2 * BUF);
    const uint32_t mine_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)mine;
    const int sdma = NATURAL ? r / 8 : 2 * RG;       // NATURAL: 64 rows x 2 r bytes = r / 8 KB

    // a row-wise load covers staged rows 8 d .. 8 d + 7; this lane: row 8 d + lane / 8, LDS slot lane % 8, which
    // receives piece slot ^ (row % 8) of the stretch
    const int d_row = lane >> 3, d_piece = (lane & 7) ^ d_row;
    uint32_t xoff[XDMA], soff[SDMA_MAX];
#pragma unroll
    for (int d = 0; d < XDMA; ++d) xoff[d] = (uint32_t)min(m0 + 8 * d + d_row, M - 1) * (uint32_t)C * 2u;
#pragma unroll
    for (int d = 0; d < SDMA_MAX; ++d)
        soff[d] = NATURAL ? (uint32_t)(d * 1024 + lane * 16)                               // within the 64-row block
                          : (uint32_t)min(8 * d + d_row, r - 1) * (uint32_t)C * 2u;        // row 8 d + lane / 8 of small
    auto fetch = [&](int col0, int buf) {
        const uint32_t cb = (uint32_t)min(col0 + 8 * d_piece, C - 8) * 2u;       // past the end: the last piece again
        const uint32_t base = mine_lds + buf * BUF;
#pragma unroll
        for (int d = 0; d < XDMA; ++d)
            dma16(act, xoff[d] + cb, (uint32_t)__builtin_amdgcn_readfirstlane((int)(base + d * 1024)));
        if constexpr (NATURAL) {
            const uint32_t blk = (uint32_t)col0 * (uint32_t)r * 2u, last = (uint32_t)C * (uint32_t)r * 2u - 16u;
#pragma unroll
            for (int d = 0; d < SDMA_MAX; ++d)
                if (d < sdma)       // wave-uniform
                    dma16(small, min(blk + soff[d], last),
                          (uint32_t)__builtin_amdgcn_readfirstlane((int)(base + SK_ROWS * 128 + d * 1024)));
        } else {
#pragma unroll
            for (int d = 0; d < SDMA_MAX; ++d)
                dma16(small, soff[d] + cb, (uint32_t)__builtin_amdgcn_readfirstlane((int)(base + (XDMA + d) * 1024)));
        }
        if constexpr (MASKED) {     // lane l: dword l % 2 of the 8 keep bytes of token row l / 2 (rows past the tile: copies)
            const uint32_t row = (uint32_t)min(m0 + min(lane >> 1, SK_ROWS - 1), M - 1);
            dma4(keep, row * (uint32_t)(C / 8) + (uint32_t)min(col0 / 8 + 4 * (lane & 1), C / 8 - 4),
                 (uint32_t)__builtin_amdgcn_readfirstlane((int)(base + MASK_OFF)));
        }
    };
    float4_t acc[RG];
    bool sval[RG];
#pragma unroll
    for (int g = 0; g < RG; ++g) {
        acc[g] = float4_t{0.f, 0.f, 0.f, 0.f};
        sval[g] = g * 16 + li < r;
    }
    // NATURAL: this lane's address within a 32-row chunk of the block, 16-column group 0 (see above)
    const int t_off = (8 * q + (li >> 2)) * (r * 2);
    auto consume = [&](int col0, int buf) {
        const char *bp = mine + buf * BUF;
#pragma unroll
        for (int cc = 0; cc < SS_COLS / 32; ++cc) {
            const int slot = (4 * cc + q) ^ (li & 7);
            const bool in = col0 + 32 * cc + 8 * q < C;
            u16x8_t xa = *(const u16x8_t *)(bp + (rowin ? li : 0) * 128 + slot * 16);
            if constexpr (MASKED) xa = keep_halves(xa, *(const uint8_t *)(bp + MASK_OFF + (rowin ? li : 0) * 8 + 4 * cc + q));
            if (!(in && rowin)) xa = u16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < RG; ++g) {
                u16x8_t sb;
                if constexpr (NATURAL) {
                    const char *ch = bp + SK_ROWS * 128 + cc * 32 * (r * 2) + t_off + 2 * min(16 * g + 4 * (li & 3), r - 4);
                    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)ch);
                    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(ch + 4 * (r * 2)));
                    sb = u16x8_t{(uint16_t)lo[0], (uint16_t)lo[1], (uint16_t)lo[2], (uint16_t)lo[3],
                                 (uint16_t)hi[0], (uint16_t)hi[1], (uint16_t)hi[2], (uint16_t)hi[3]};
                    if (!(in && sval[g])) sb = u16x8_t{0, 0, 0, 0, 0, 0, 0, 0};   // rows past C hold copies of valid data
                } else {
                    sb = *(const u16x8_t *)(bp + (SK_ROWS + 16 * g + li) * 128 + slot * 16);
                    if (!sval[g]) sb = u16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                }
                acc[g] = mfma16<BF16>(xa, sb, acc[g]);
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");          // the buffer is read out before it is refilled
    };
    constexpr int STEP = SK_WAVES * SS_COLS;
    const int loads = XDMA + sdma + (MASKED ? 1 : 0);               // per stretch
    int col0 = wave * SS_COLS, buf = 0;
    if (col0 < C) fetch(col0, 0);
    if (col0 + STEP < C) fetch(col0 + STEP, 1);
    for (; col0 < C; col0 += STEP, buf ^= 1) {
        // the stretch in `buf` was requested before the one in the other buffer (if there is one): leave only the
        // younger stretch's loads in flight (the count is wave-uniform; the instruction needs it as an immediate)
        if (col0 + STEP < C) {
            switch (loads) {
            case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
            case 3: asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); break;
            case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
            case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
            case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
            case 7: asm volatile("s_waitcnt vmcnt(7)" ::: "memory"); break;
            case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
            case 9: asm volatile("s_waitcnt vmcnt(9)" ::: "memory"); break;
            case 10: asm volatile("s_waitcnt vmcnt(10)" ::: "memory"); break;
            case 11: asm volatile("s_waitcnt vmcnt(11)" ::: "memory"); break;
            default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;   // stricter than needed, never laxer
            }
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        consume(col0, buf);
        if (col0 + 2 * STEP < C) fetch(col0 + 2 * STEP, buf);
    }
    __syncthreads();                                                // every wave is done with its buffers
    float(*red)[RG][16][17] = reinterpret_cast<float(*)[RG][16][17]>(ss_lds);   // [SK_WAVES][RG][16][17]
#pragma unroll
    for (int g = 0; g < RG; ++g)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][g][4 * q + v][li] = acc[g][v];
    __syncthreads();
    for (int e = threadIdx.x; e < RG * 256; e += SK_WAVES * 64) {
        const int g = e >> 8, row = (e >> 4) & 15, col = e & 15;
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < SK_WAVES; ++w) s += red[w][g][row][col];
        if constexpr (MASKED) s *= keep_scale;
        if (row < SK_ROWS && m0 + row < M && g * 16 + col < r) out[(long)(m0 + row) * r + g * 16 + col] = to16<BF16>(s);
    }
}

// Arguments of the adapter-gradient launch: dB (problem 0: act = dY, side = t) and dA (problem 1: act = x, side = u).
struct GradArgs {
    const uint16_t *act[2], *side[2];
    float *out[2];          // dB [C0, r] and dA [r, C1]
    int C[2];
    int nb0;                // column blocks of the first problem
    int M, r;               // r: adapter columns the gradients are formed for
    int side_pitch, side_c0;   // side is [M, side_pitch]; its columns side_c0 .. side_c0 + r are used (stacked adapters:
                               // the leading side_c0 columns belong to a frozen pair)
    float sc[2], beta;      // out = beta * out + sc * sum (beta == 0: out is not read)
    const uint8_t *keep;    // LoRA dropout: keep bits of x (the second problem's act), [M, C1/8] bytes, or NULL
};

// ------------------------------------------------------------------------------------------------------------
// dB and dA in one pass, without slice partial sums (ranks <= 16, no dropout mask): a workgroup owns 32 columns of
// dY (for dB) or x (for dA) and walks all token rows.  Each of its eight waves takes 64-row stretches (wave w the
// stretches w, w + 8, ...): it pulls the stretch of its 32 columns (64 bytes per row) and of the side operand (t or
// u, its trainable columns) into one of two wave-private LDS buffers with direct-to-LDS loads -- the next stretch is
// in flight while this one is multiplied, the wave waits on its own loads, no workgroup barrier in the loop -- and
// gathers both MFMA operands (the contraction runs over the row index, the strided one) with the transposing LDS
// read.  The eight partial results are added in wave order at the end and written as out = beta * out + sc * sum.
// Measured at 2048 x (4096 + 4096), rank 8: 8.2 us against 9.9 + 4.7 us for the slice sums and their reduction.
// ------------------------------------------------------------------------------------------------------------
constexpr int GO_COLS = 32, GO_WAVES = 8;
constexpr int go_rows(int R) { return R <= 32 ? 64 : 32; }                   // rows per stretch
constexpr int go_buf_bytes(int R) { return go_rows(R) * (GO_COLS + (R < 16 ? 16 : R)) * 2 + 256; }   // activations + side + mask
constexpr int go_lds_bytes(int R)
{
    const int pipe = GO_WAVES * 2 * go_buf_bytes(R), sum = GO_WAVES * ((R + 15) / 16 * 16) * GO_COLS * 4;
    return pipe > sum ? pipe : sum;
}
// R: side columns staged per row, 8, 16, 32 or 64; the rank a.r may be smaller (24 in 32; 40, 48, 56 in 64): the
// missing 8-column pieces are fetched as copies of the last one and count as zero.  MASKED: a.keep != NULL
template <bool BF16, int R, bool MASKED>
__global__ __launch_bounds__(GO_WAVES * 64) void adapter_grad_onepass_kernel(const GradArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char go_lds[];   // [GO_WAVES][2] buffers, then reused for the final sum
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4_t *lds4_t;
    constexpr int GO_ROWS = go_rows(R), GO_ACT_BYTES = GO_ROWS * GO_COLS * 2, GO_BUF_BYTES = go_buf_bytes(R);
    constexpr int GO_MASK_OFF = GO_BUF_BYTES - 256;          // LoRA dropout: the 32 keep bits of each row of the stretch
    constexpr int RG = (R + 15) / 16;                        // 16-column groups of the side operand
    constexpr int PR = R / 8, S_ROWS = 64 / PR;              // 16-byte pieces per side row; side rows per load
    constexpr int LOADS = GO_ROWS / 16 + GO_ROWS / S_ROWS;   // direct-to-LDS loads per stretch
    static_assert(GO_ROWS % S_ROWS == 0 && GO_ROWS % 32 == 0, "whole loads and whole chunks per stretch");
    // Consecutive workgroup ids land on different XCDs; a 32-column block is half a 128-byte line per row, so each
    // XCD is handed a contiguous run of column blocks: both halves of a line are then fetched through the same L2.
    int blk;
    {
        const int nt = gridDim.x, bid = blockIdx.x;
        const int xcd = bid & 7, loc = bid >> 3, per = nt >> 3, rem = nt & 7;
        blk = xcd * per + min(xcd, rem) + loc;
    }
    const int which = blk >= a.nb0 ? 1 : 0;
    const uint16_t *__restrict__ act = a.act[which];
    const uint16_t *__restrict__ side = a.side[which];
    const int M = a.M, C = a.C[which];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int c0 = (blk - (which ? a.nb0 : 0)) * GO_COLS;
    const int li = lane & 15, q = lane >> 4;
    char *mine = go_lds + wave * (2 * GO_BUF_BYTES);
    const uint32_t mine_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)mine;

    // what this lane fetches: of the activations, piece lane % 4 (8 columns) of row lane / 4 of every 16-row block;
    // of the side operand, piece lane % PR of row lane / PR of every S_ROWS-row block
    const int a_row = lane >> 2, a_col = min(c0 + 8 * (lane & 3), C - 8);
    const int r = a.r;                                       // r <= R, r % 8 == 0
    const int s_row = lane / PR, s_col = a.side_c0 + 8 * min(lane % PR, r / 8 - 1);
    // transposing reads (see skinny_rows_staged_kernel): lane (e = li / 4, g = li % 4) of block q points at row
    // 8 q + e, columns 4 g .. + 4 of a 32-row chunk; the second read of a fragment starts four rows further down
    const int t_row = 8 * q + (li >> 2);
    const int act_rd = t_row * (GO_COLS * 2) + 8 * (li & 3);                      // + 32 for the second 16 columns
    const int side_rd = GO_ACT_BYTES + t_row * (R * 2) + 2 * min(4 * (li & 3), R - 4);   // + 32 per 16-column group

    // this wave's stretches: rows (GO_WAVES i + wave) * GO_ROWS .. + GO_ROWS, i = 0, 1, ...; two are in flight
    auto fetch = [&](int m0, int buf) {
        const uint32_t base = mine_lds + buf * GO_BUF_BYTES;
#pragma unroll
        for (int b = 0; b < GO_ROWS / 16; ++b) {
            const uint32_t row = (uint32_t)min(m0 + 16 * b + a_row, M - 1);     // past the end: copies of the last row
            dma16(act, (row * (uint32_t)C + (uint32_t)a_col) * 2u,
                  (uint32_t)__builtin_amdgcn_readfirstlane((int)(base + b * 1024)));
        }
#pragma unroll
        for (int b = 0; b < GO_ROWS / S_ROWS; ++b) {
            const uint32_t row = (uint32_t)min(m0 + S_ROWS * b + s_row, M - 1);
            dma16(side, (row * (uint32_t)a.side_pitch + (uint32_t)s_col) * 2u,
                  (uint32_t)__builtin_amdgcn_readfirstlane((int)(base + GO_ACT_BYTES + b * 1024)));
        }
        if (MASKED && which) {      // dA sees keep_scale * x * keep: lane l fetches the keep bits of row l, columns c0 .. c0 + 32
            const uint32_t row = (uint32_t)min(m0 + lane, M - 1);
            dma4(a.keep, row * (uint32_t)(C / 8) + (uint32_t)(c0 / 8),
                 (uint32_t)__builtin_amdgcn_readfirstlane((int)(base + GO_MASK_OFF)));
        }
    };
    float4_t acc[RG][2];
#pragma unroll
    for (int g = 0; g < RG; ++g) acc[g][0] = acc[g][1] = float4_t{0.f, 0.f, 0.f, 0.f};
    auto consume = [&](int m0, int buf) {
        const char *bp = mine + buf * GO_BUF_BYTES;
        const int rows_here = min(GO_ROWS, M - m0);
#pragma unroll
        for (int ch = 0; ch < GO_ROWS / 32; ++ch) {
            u16x8_t fb[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const s16x4_t x_lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(bp + act_rd + ch * 32 * (GO_COLS * 2) + 32 * h));
                const s16x4_t x_hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(bp + act_rd + (ch * 32 + 4) * (GO_COLS * 2) + 32 * h));
                fb[h] = u16x8_t{(uint16_t)x_lo[0], (uint16_t)x_lo[1], (uint16_t)x_lo[2], (uint16_t)x_lo[3],
                                (uint16_t)x_hi[0], (uint16_t)x_hi[1], (uint16_t)x_hi[2], (uint16_t)x_hi[3]};
            }
            if (MASKED && which) {  // this lane holds column 16 h + li of rows 8 q .. 8 q + 7 of the chunk
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t bits = *(const uint32_t *)(bp + GO_MASK_OFF + (ch * 32 + 8 * q + e) * 4);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        if (!((bits >> (16 * h + li)) & 1u)) fb[h][e] = 0;
                }
            }
            const int left = rows_here - (ch * 32 + 8 * q);         // valid rows among this lane's eight
#pragma unroll
            for (int g = 0; g < RG; ++g) {
                const s16x4_t s_lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(bp + side_rd + ch * 32 * (R * 2) + 32 * g));
                const s16x4_t s_hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(bp + side_rd + (ch * 32 + 4) * (R * 2) + 32 * g));
                u16x8_t fa = {(uint16_t)s_lo[0], (uint16_t)s_lo[1], (uint16_t)s_lo[2], (uint16_t)s_lo[3],
                              (uint16_t)s_hi[0], (uint16_t)s_hi[1], (uint16_t)s_hi[2], (uint16_t)s_hi[3]};
                // rows past M were fetched as copies of the last row: their side values count as zero; so do the
                // columns past the rank
                const bool jval = 16 * g + li < r;
                if (!jval || left < 8) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (!jval || e >= left) fa[e] = 0;
                }
#pragma unroll
                for (int h = 0; h < 2; ++h) acc[g][h] = mfma16<BF16>(fa, fb[h], acc[g][h]);   // D[j = 16 g + 4 q + v][c = 16 h + li]
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");          // the buffer is read out before it is refilled
    };
    constexpr int STEP = GO_WAVES * GO_ROWS;
    int m0 = wave * GO_ROWS, buf = 0;
    if (m0 < M) fetch(m0, 0);
    if (m0 + STEP < M) fetch(m0 + STEP, 1);
    for (; m0 < M; m0 += STEP, buf ^= 1) {
        // the stretch in `buf` was requested before the one in the other buffer (if there is one)
        if (m0 + STEP >= M) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else if (MASKED && which) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS + 1) : "memory");   // + the keep bits
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LOADS) : "memory");
        consume(m0, buf);
        if (m0 + 2 * STEP < M) fetch(m0 + 2 * STEP, buf);
    }
    __syncthreads();                                                // every wave is done with its buffers
    float *red = reinterpret_cast<float *>(go_lds);                 // [GO_WAVES][16 RG rows j][32 c]
#pragma unroll
    for (int g = 0; g < RG; ++g)
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                red[(wave * (16 * RG) + 16 * g + 4 * q + v) * GO_COLS + 16 * h + li] = acc[g][h][v];
    __syncthreads();
    for (int e = threadIdx.x; e < r * GO_COLS; e += GO_WAVES * 64) {
        const int j = e / GO_COLS, c = e % GO_COLS;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < GO_WAVES; ++w) sum += red[(w * (16 * RG) + j) * GO_COLS + c];
        if (c0 + c < C) {
            float *dst = a.out[which] + (which ? (long)j * C + c0 + c : (long)(c0 + c) * r + j);
            *dst = a.beta == 0.f ? a.sc[which] * sum : fmaf(a.beta, *dst, a.sc[which] * sum);
        }
    }
}

template <bool BF16, int R, bool MASKED>
void launch_grad_onepass_masked(const GradArgs &a, int blocks, hipStream_t s)
{
    constexpr int lds = go_lds_bytes(R);
    auto kern = adapter_grad_onepass_kernel<BF16, R, MASKED>;
    ensure_dynamic_lds((const void *)kern, (int)(lds));
    QLORA_LAUNCH(kern, dim3(blocks), dim3(GO_WAVES * 64), lds, s, a);
}

template <bool BF16, int R>
void launch_grad_onepass(const GradArgs &a, int blocks, hipStream_t s)
{
    if (a.keep) launch_grad_onepass_masked<BF16, R, true>(a, blocks, s);
    else launch_grad_onepass_masked<BF16, R, false>(a, blocks, s);
}

template <bool BF16, int RG, int SK_ROWS, bool NATURAL, bool MASKED>
void launch_skinny_staged(const uint16_t *act, const uint16_t *small, uint16_t *out, int M, int C, int r,
                          const uint8_t *keep, float keep_scale, hipStream_t s)
{
    constexpr int pipe = SK_WAVES * 2 * ss_buf_bytes<RG, SK_ROWS, NATURAL, MASKED>(), sum = SK_WAVES * RG * 16 * 17 * 4;
    static_assert(pipe <= 160 * 1024, "fits the LDS of a CU");
    constexpr int lds = pipe > sum ? pipe : sum;
    auto kern = skinny_rows_staged_kernel<BF16, RG, SK_ROWS, NATURAL, MASKED>;
    ensure_dynamic_lds((const void *)kern, (int)(lds));
    QLORA_LAUNCH(kern, dim3((M + SK_ROWS - 1) / SK_ROWS), dim3(SK_WAVES * 64), lds, s, act, small, out, M, C, r, keep,
                       keep_scale);
}

template <bool BF16, int SK_ROWS, bool NATURAL, bool MASKED>
void launch_skinny_staged_rank(const uint16_t *act, const uint16_t *small, uint16_t *out, int M, int C, int r,
                               const uint8_t *keep, float keep_scale, hipStream_t s)
{
    switch ((r + 15) / 16) {
    case 1: launch_skinny_staged<BF16, 1, SK_ROWS, NATURAL, MASKED>(act, small, out, M, C, r, keep, keep_scale, s); break;
    case 2: launch_skinny_staged<BF16, 2, SK_ROWS, NATURAL, MASKED>(act, small, out, M, C, r, keep, keep_scale, s); break;
    case 3: launch_skinny_staged<BF16, 3, SK_ROWS, NATURAL, MASKED>(act, small, out, M, C, r, keep, keep_scale, s); break;
    default:    // (masked, 16 rows, four rank groups do not fit the LDS: launch_skinny keeps that case away)
        if constexpr (!(MASKED && SK_ROWS == 16))
            launch_skinny_staged<BF16, 4, SK_ROWS, NATURAL, MASKED>(act, small, out, M, C, r, keep, keep_scale, s);
        break;
    }
}

template <bool BF16, bool MASKED>
void launch_skinny(const uint16_t *act, const uint16_t *small, uint16_t *out, int M, int C, int r, const uint8_t *keep,
                   float keep_scale, hipStream_t s)
{
    // 16 token rows per workgroup once that fills the chip; under a mask, 16 rows and ranks above 48 together exceed
    // the LDS, so those keep 8-row workgroups
    if (M >= 16 * 256 && !(MASKED && r > 48))
        launch_skinny_staged_rank<BF16, 16, false, MASKED>(act, small, out, M, C, r, keep, keep_scale, s);
    else
        launch_skinny_staged_rank<BF16, 8, false, MASKED>(act, small, out, M, C, r, keep, keep_scale, s);
}

// ---- t = x A^T for up to 32 token rows.  The kernel above gives a workgroup eight token rows and the whole
//      contraction: at 16 rows that is two workgroups, each pulling all of A through one compute unit (8 us at K = 4096,
//      rank 40).  Here the contraction is split instead: workgroup p multiplies columns [p chunk, (p + 1) chunk), its
//      four waves taking 32-column steps in turn, and leaves an fp32 plane [M][r]; a second, tiny launch sums the planes
//      in order and rounds once.
template <bool BF16>
__global__ __launch_bounds__(256) void lora_down_small_partial_kernel(const uint16_t *__restrict__ x,
                                                                      const uint16_t *__restrict__ A,
                                                                      float *__restrict__ part, int M, int K, int r,
                                                                      int chunk)
{
    __shared__ float red[4][2][4][16][17];             // [wave][token block][rank block][m][j]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, li = lane & 15, q = lane >> 4;
    const int k_begin = (int)blockIdx.x * chunk, k_end = min(K, k_begin + chunk);
    const int mbs = (M + 15) / 16, rgs = (r + 15) / 16;                       // at most 2 and 4
    const u16x8_t ZERO8 = {0, 0, 0, 0, 0, 0, 0, 0};
    float4_t acc[2][4];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g) acc[b][g] = float4_t{0.f, 0.f, 0.f, 0.f};
    for (int k0 = k_begin + 32 * wave; k0 < k_end; k0 += 128) {             // K is a multiple of 32: whole steps
        u16x8_t xf[2], af[4];
#pragma unroll
        for (int b = 0; b < 2; ++b)
            xf[b] = b < mbs ? *(const u16x8_t *)(x + (long)min(16 * b + li, M - 1) * K + k0 + 8 * q) : ZERO8;
#pragma unroll
        for (int g = 0; g < 4; ++g)
            af[g] = (g < rgs && 16 * g + li < r) ? *(const u16x8_t *)(A + (long)(16 * g + li) * K + k0 + 8 * q) : ZERO8;
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g)
                if (b < mbs && g < rgs) acc[b][g] = mfma16<BF16>(xf[b], af[g], acc[b][g]);   // D[m = 4q+v][j = li]
    }
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][b][g][4 * q + v][li] = acc[b][g][v];
    __syncthreads();
    float *plane = part + (size_t)blockIdx.x * M * r;
    for (int e = threadIdx.x; e < M * r; e += 256) {
        const int m = e / r, j = e % r;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) v += red[w][m >> 4][j >> 4][m & 15][j & 15];
        plane[e] = v;
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void lora_down_small_sum_kernel(const float *__restrict__ part,
                                                                  uint16_t *__restrict__ t, int planes, int count)
{
    const int e = (int)blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    float v = 0.f;
    for (int p0 = 0; p0 < planes; p0 += 16) {           // sixteen planes requested together, summed in plane order
        float pv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) pv[i] = p0 + i < planes ? part[(size_t)(p0 + i) * count + e] : 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) v += pv[i];
    }
    t[e] = to16<BF16>(v);
}

}  // namespace

int lora_down_small_chunk(int K)
{
    const int c = (K / 64 + 127) / 128 * 128;          // about 64 planes at most, whole steps of the four waves
    return c < 128 ? 128 : c;
}
int lora_down_small_planes(int K) { return (K + lora_down_small_chunk(K) - 1) / lora_down_small_chunk(K); }

void launch_lora_down(const void *x, const void *A, void *t, int M, int K, int r, bool bf16, const uint32_t *keep,
                      float keep_scale, hipStream_t s, float *planes)
{
    const uint16_t *xp = (const uint16_t *)x, *Ap = (const uint16_t *)A;
    uint16_t *tp = (uint16_t *)t;
    const uint8_t *kb = (const uint8_t *)keep;
    if (planes && !keep && M <= LORA_DOWN_SMALL_MAX_M) {
        const int chunk = lora_down_small_chunk(K), np = lora_down_small_planes(K);
        const dim3 sum_grid((unsigned)((M * r + 255) / 256));
        if (bf16) {
            QLORA_LAUNCH(lora_down_small_partial_kernel<true>, dim3(np), dim3(256), 0, s, xp, Ap, planes, M, K, r, chunk);
            QLORA_LAUNCH(lora_down_small_sum_kernel<true>, sum_grid, dim3(256), 0, s, planes, tp, np, M * r);
        } else {
            QLORA_LAUNCH(lora_down_small_partial_kernel<false>, dim3(np), dim3(256), 0, s, xp, Ap, planes, M, K, r, chunk);
            QLORA_LAUNCH(lora_down_small_sum_kernel<false>, sum_grid, dim3(256), 0, s, planes, tp, np, M * r);
        }
        return;
    }
    if (keep) {
        if (bf16) launch_skinny<true, true>(xp, Ap, tp, M, K, r, kb, keep_scale, s);
        else launch_skinny<false, true>(xp, Ap, tp, M, K, r, kb, keep_scale, s);
    } else {
        if (bf16) launch_skinny<true, false>(xp, Ap, tp, M, K, r, nullptr, 1.f, s);
        else launch_skinny<false, false>(xp, Ap, tp, M, K, r, nullptr, 1.f, s);
    }
}

void launch_lora_u(const void *dy, const void *B, void *u, int M, int N, int r, bool bf16, hipStream_t s)
{
    const uint16_t *a = (const uint16_t *)dy, *b = (const uint16_t *)B;
    uint16_t *o = (uint16_t *)u;
    // B is read as it lies in memory (the contraction index is its strided one: transposing LDS reads)
    if (M >= 16 * 256) {
        if (bf16) launch_skinny_staged_rank<true, 16, true, false>(a, b, o, M, N, r, nullptr, 1.f, s);
        else launch_skinny_staged_rank<false, 16, true, false>(a, b, o, M, N, r, nullptr, 1.f, s);
    } else {
        if (bf16) launch_skinny_staged_rank<true, 8, true, false>(a, b, o, M, N, r, nullptr, 1.f, s);
        else launch_skinny_staged_rank<false, 8, true, false>(a, b, o, M, N, r, nullptr, 1.f, s);
    }
}

// dX[m,k] += f[m,k] * sum_j u[m,j] A[j,k],  f = sc * keep_scale where the keep bit of (m,k) is set, else 0:
// the adapter's share of dX under LoRA dropout, added to the base product the GEMM left in dX (which then carried
// no adapter steps).  A workgroup owns 64 rows x 256 columns; u and the A columns are staged in LDS.
template <bool BF16>
__global__ __launch_bounds__(256) void lora_dx_masked_kernel(uint16_t *__restrict__ dx, const uint16_t *__restrict__ u,
                                                             const uint16_t *__restrict__ A,
                                                             const uint8_t *__restrict__ keep, int M, int K, int r,
                                                             float f)
{
    __shared__ float us[64][64 + 1];
    __shared__ uint16_t As[64][256 + 8];
    const int m0 = blockIdx.y * 64, k0 = blockIdx.x * 256, tid = threadIdx.x;
    for (int e = tid; e < 64 * r; e += 256) {
        const int m = e / r, j = e % r;
        us[m][j] = m0 + m < M ? cvt16<BF16>(u[(long)(m0 + m) * r + j]) : 0.f;
    }
    for (int e = tid; e < r * 32; e += 256) {              // A rows of this column block, 8 columns at a time
        const int j = e >> 5, c = (e & 31) * 8;
        u16x8_t v = u16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
        if (k0 + c < K) v = *(const u16x8_t *)(A + (long)j * K + k0 + c);
        *(u16x8_t *)&As[j][c] = v;
    }
    __syncthreads();
    const int c = (tid & 31) * 8;                          // this thread's 8 columns; rows tid/32, +8, ...
    if (k0 + c >= K) return;
    for (int m = tid >> 5; m < 64 && m0 + m < M; m += 8) {
        uint16_t *p = dx + (long)(m0 + m) * K + k0 + c;
        u16x8_t d = *(const u16x8_t *)p;
        const uint32_t kb = keep[(long)(m0 + m) * (K / 8) + ((k0 + c) >> 3)];
        float lo[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) lo[e] = 0.f;
        for (int j = 0; j < r; ++j) {
            const float uj = us[m][j];
            const u16x8_t av = *(const u16x8_t *)&As[j][c];
#pragma unroll
            for (int e = 0; e < 8; ++e) lo[e] = fmaf(uj, cvt16<BF16>(av[e]), lo[e]);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if ((kb >> e) & 1u) d[e] = to16<BF16>(fmaf(f, lo[e], cvt16<BF16>(d[e])));
        *(u16x8_t *)p = d;
    }
}

void launch_lora_dx_masked(void *dx, const void *u, const void *A, const uint32_t *keep, int M, int K, int r, float f,
                           bool bf16, hipStream_t s)
{
    const dim3 grid((K + 255) / 256, (M + 63) / 64), block(256);
    if (bf16)
        QLORA_LAUNCH(lora_dx_masked_kernel<true>, grid, block, 0, s, (uint16_t *)dx, (const uint16_t *)u,
                           (const uint16_t *)A, (const uint8_t *)keep, M, K, r, f);
    else
        QLORA_LAUNCH(lora_dx_masked_kernel<false>, grid, block, 0, s, (uint16_t *)dx, (const uint16_t *)u,
                           (const uint16_t *)A, (const uint8_t *)keep, M, K, r, f);
}

void launch_adapter_grads(const void *dy, const void *t, const void *x, const void *u, float *dB, float *dA, int M, int N,
                          int K, int r_all, int frozen, float sc, float beta, const uint32_t *keep, float keep_scale,
                          bool bf16, hipStream_t s)
{
    const int r = r_all - frozen;
    GradArgs a;
    a.act[0] = (const uint16_t *)dy;
    a.side[0] = (const uint16_t *)t;
    a.act[1] = (const uint16_t *)x;
    a.side[1] = (const uint16_t *)u;
    a.out[0] = dB;
    a.out[1] = dA;
    a.C[0] = N;
    a.C[1] = K;
    a.nb0 = (N + GO_COLS - 1) / GO_COLS;
    a.M = M;
    a.r = r;
    a.side_pitch = r_all;
    a.side_c0 = frozen;
    a.sc[0] = sc;
    a.sc[1] = keep ? sc * keep_scale : sc;
    a.beta = beta;
    a.keep = (const uint8_t *)keep;
    // ranks 24, 40, 48 and 56 run in the next larger of the kernel's side widths 8, 16, 32, 64
    const int blocks = a.nb0 + (K + GO_COLS - 1) / GO_COLS;
#define QLORA_ONEPASS(R)                                       \
    do {                                                       \
        if (bf16) launch_grad_onepass<true, R>(a, blocks, s);  \
        else launch_grad_onepass<false, R>(a, blocks, s);      \
        return;                                                \
    } while (0)
    if (r == 8) QLORA_ONEPASS(8);
    if (r == 16) QLORA_ONEPASS(16);
    if (r <= 32) QLORA_ONEPASS(32);
    QLORA_ONEPASS(64);
#undef QLORA_ONEPASS
}

}  // namespace qlora
