// Tiled MFMA GEMM over the packed weight with dequantisation fused into the operand staging.
//
//   forward   (TRANS = false):  y [M,N]  = x [M,K]  * Wd[N,K]^T  + sc * t[M,r] * B[N,r]^T      (Fig. 1, forward path)
//   backward  (TRANS = true):   dX[M,K]  = dY[M,N]  * Wd[N,K]    + sc * u[M,r] * A[r,K]        (Sec. 3.1: the packed
//             weight is consumed transposed; transpose + unpack + matmul happen inside this one kernel)
//
// Both are C[M,NO] = Act[M,KC] * W^T with W viewed as [NO,KC]; only the way a packed tile is fetched and laid
// into LDS differs.  A workgroup of 4 waves owns a BM x BN output tile and walks the contraction in steps of
// 64: activation chunks go global -> registers -> LDS unchanged, packed words go global -> registers ->
// (unpack, s*(q-z), round to 16 bit) -> LDS, and v_mfma_f32_32x32x16 consumes 16-byte fragments from LDS.
// The dequantised weight never reaches HBM.  The rank-r LoRA term is folded in as extra contraction steps.
#include "common.hpp"
#include "dequant.hpp"
#include "kernels.hpp"

namespace qlora {

namespace {

constexpr int BK = 64;               // contraction elements per LDS stage
constexpr int LDS_STRIDE = BK + 8;   // 144-byte rows: the 16-byte reads of 8 consecutive rows fall in distinct bank groups
constexpr int THREADS = 256;

struct GemmArgs {
    const uint16_t *act;      // x (forward) or dY (backward): [M, KC]
    const uint32_t *packed;   // [N, K*BITS/32]
    const uint16_t *scales;   // fp16 [N, K/G]
    const uint8_t *zeros;     // [N, K/G]
    const uint16_t *ext_act;  // t (forward) or u (backward): [M, r]; unused when r == 0
    const uint16_t *ext_w;    // B [N,r] (forward) or A [r,K] (backward)
    uint16_t *out;            // y [M,N] or dX [M,K]
    int M, N, K, G, r;
    float sc;
    int tiles_m, tiles_n;
    uint32_t g32_magic;       // see group_magic(): (k/32) / (G/32) == umulhi(k/32, magic), 0 meaning G == 32
};

template <bool BF16>
__device__ __forceinline__ float16_t mfma32(u16x8_t a, u16x8_t b, float16_t c)
{
    if constexpr (BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                       c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c,
                                                      0, 0, 0);
}

// 32 consecutive codes of one row are exactly BITS words.
template <int BITS>
__device__ __forceinline__ void load_unit(const uint32_t *__restrict__ p, uint32_t (&w)[BITS])
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

// What one thread fetches for one 64-deep stage: XCH activation chunks and WU packed units with their group's
// scale and zero-point.
template <int BITS, int XCH, int WU>
struct StageRegs {
    u32x4_t x[XCH];
    uint32_t w[WU][BITS];
    float s[WU], z[WU];
};

template <int BITS, bool BF16, bool TRANS, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(THREADS) void qgemm_kernel(const GemmArgs a)
{
    static_assert(WM * WN == 4, "four waves per workgroup");
    static_assert(BN % 128 == 0 && BM % 128 == 0, "tile shape");
    constexpr int TM = BM / WM, TN = BN / WN;       // per-wave output tile
    constexpr int MI = TM / 32, NI = TN / 32;       // 32x32 MFMA blocks per wave
    constexpr int XCH = BM * (BK / 8) / THREADS;    // 16-byte activation chunks per thread per stage
    constexpr int WU = BN / 128;                    // 32-code weight units per thread per stage
    constexpr int STAGE = (BM + BN) * LDS_STRIDE;   // halfs per LDS stage
    constexpr int KSTEPS = BK / 16;                 // MFMA k-steps per stage
    using Regs = StageRegs<BITS, XCH, WU>;

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int NO = TRANS ? a.K : a.N;    // output columns
    const int KC = TRANS ? a.N : a.K;    // contraction length
    const int ng = a.K / a.G, Kw = a.K * BITS / 32;

    // --- which tile: consecutive workgroups land on different XCDs, so hand each XCD a contiguous run of tile
    //     ids, and order ids so that a run covers a compact block of tiles (shared rows and columns hit in L2)
    int pm, pn;
    {
        const int nt = a.tiles_m * a.tiles_n, bid = blockIdx.x;
        const int xcd = bid & 7, loc = bid >> 3, per = nt >> 3, rem = nt & 7;
        const int t = xcd * per + min(xcd, rem) + loc;
        constexpr int GM = 4;
        const int in_group = GM * a.tiles_n, group = t / in_group, first_m = group * GM;
        const int gsz = min(a.tiles_m - first_m, GM), o = t % in_group;
        pm = first_m + o % gsz;
        pn = o / gsz;
    }
    const int row0 = pm * BM, col0 = pn * BN;

    float16_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // global -> registers for stage kt.  Branch-free: every address is clamped into the valid range and whatever
    // lies beyond the contraction length (or beyond the weight's rows / columns) is neutralised by a zero scale
    // on the weight side, so stages past the end may be fetched and staged harmlessly.
    const uint32_t xkc = (tid & 7) * 8;                 // same k offset for every chunk of this thread
    uint32_t xrow_off[XCH];                             // element offset of each chunk's row
#pragma unroll
    for (int i = 0; i < XCH; ++i) xrow_off[i] = (uint32_t)min(row0 + ((tid + THREADS * i) >> 3), a.M - 1) * (uint32_t)KC;

    auto load_global = [&](int kt, Regs &rg) {
        const int kbase = kt * BK;
        const uint32_t k = (uint32_t)min(kbase + (int)xkc, KC - 8);
#pragma unroll
        for (int i = 0; i < XCH; ++i) rg.x[i] = *(const u32x4_t *)(a.act + (xrow_off[i] + k));
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const int u = tid + THREADS * i;
            int n, k0;
            bool ok;
            if constexpr (TRANS) {          // 64 contraction rows n, BN/32 units across the output columns k
                n = kbase + (u & 63);
                k0 = col0 + (u >> 6) * 32;
                ok = n < a.N && k0 < a.K;
            } else {                        // BN output rows n, 2 units along the contraction k
                n = col0 + (u >> 1);
                k0 = kbase + (u & 1) * 32;
                ok = k0 < a.K;
            }
            n = min(n, a.N - 1);
            k0 = min(k0, a.K - 32);
            load_unit<BITS>(a.packed + (long)n * Kw + (k0 >> 5) * BITS, rg.w[i]);
            const long gi = (long)n * ng + (a.g32_magic ? (int)__umulhi((uint32_t)(k0 >> 5), a.g32_magic) : (k0 >> 5));
            const float sv = f16_bits_to_f32(a.scales[gi]);
            rg.s[i] = ok ? sv : 0.f;
            rg.z[i] = (float)a.zeros[gi];
        }
    };

    // registers -> LDS, quarter `part` of a stage: XCH/4 activation chunks, and 8 codes of every unit dequantised
    auto stage_part = [&](const Regs &rg, const DequantConst<BITS, BF16> (&dq)[WU], int part, int buf) {
        uint16_t *As = smem + buf * STAGE, *Bs = As + BM * LDS_STRIDE;
#pragma unroll
        for (int ii = 0; ii < XCH / KSTEPS; ++ii) {
            const int i = part * (XCH / KSTEPS) + ii;
            const int c = tid + THREADS * i, r = c >> 3, kc = (c & 7) * 8;
            *(u32x4_t *)(As + r * LDS_STRIDE + kc) = rg.x[i];
        }
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const int u = tid + THREADS * i;
            const u16x8_t v = dequant8<BITS, BF16>(rg.w[i], part, dq[i]);
            if constexpr (TRANS) {
                uint16_t *dst = Bs + ((u >> 6) * 32 + part * 8) * LDS_STRIDE + (u & 63);
#pragma unroll
                for (int e = 0; e < 8; ++e) dst[e * LDS_STRIDE] = v[e];
            } else {
                *(u16x8_t *)(Bs + (u >> 1) * LDS_STRIDE + (u & 1) * 32 + part * 8) = v;
            }
        }
    };

    struct Frags {
        u16x8_t a[MI], b[NI];
    };
    const int fr = lane & 31, fk = (lane >> 5) * 8;
    auto load_frags = [&](int buf, int ks, Frags &f) {
        const uint16_t *As = smem + buf * STAGE, *Bs = As + BM * LDS_STRIDE;
#pragma unroll
        for (int i = 0; i < MI; ++i) f.a[i] = *(const u16x8_t *)(As + (wm * TM + i * 32 + fr) * LDS_STRIDE + ks * 16 + fk);
#pragma unroll
        for (int j = 0; j < NI; ++j) f.b[j] = *(const u16x8_t *)(Bs + (wn * TN + j * 32 + fr) * LDS_STRIDE + ks * 16 + fk);
    };
    auto mfma_frags = [&](const Frags &f) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) acc[i][j] = mfma32<BF16>(f.a[i], f.b[j], acc[i][j]);
    };

    // One stage of the pipeline: MFMAs on LDS buffer kt&1 interleaved with staging stage kt+1 (held in `next`)
    // into the other buffer, while stage kt+2 is fetched from memory into `fetch`.  Identical for every kt.
    const int KT = (KC + BK - 1) / BK;
    auto pipeline_step = [&](int kt, const Regs &next, Regs &fetch) {
        load_global(kt + 2, fetch);     // `fetch` held stage kt, which was staged during the previous step
        DequantConst<BITS, BF16> dq[WU];
#pragma unroll
        for (int i = 0; i < WU; ++i) dq[i].set(next.s[i], next.z[i]);
        Frags f[2];
        load_frags(kt & 1, 0, f[0]);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            if (ks + 1 < KSTEPS) load_frags(kt & 1, ks + 1, f[(ks + 1) & 1]);
            stage_part(next, dq, ks, (kt + 1) & 1);
            mfma_frags(f[ks & 1]);
        }
        __syncthreads();
    };

    Regs r0, r1;
    load_global(0, r0);
    load_global(1, r1);
    {
        DequantConst<BITS, BF16> dq[WU];
#pragma unroll
        for (int i = 0; i < WU; ++i) dq[i].set(r0.s[i], r0.z[i]);
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) stage_part(r0, dq, ks, 0);
    }
    __syncthreads();
    for (int kt = 0; kt < KT; kt += 2) {
        pipeline_step(kt, r1, r0);
        if (kt + 1 < KT) pipeline_step(kt + 1, r0, r1);
    }

    // --- LoRA term as extra contraction steps: Act' = sc * t (or u), W' = B (or A^T), zero-padded to 16
    if (a.r > 0) {
        const int nsteps = (a.r + 15) / 16, width = nsteps * 16;
        uint16_t *As = smem, *Bs = As + BM * LDS_STRIDE;
        const int cpr = width / 8;                      // 8-element chunks per row
        for (int c = tid; c < BM * cpr; c += THREADS) {
            const int r = c / cpr, j = (c % cpr) * 8;
            u16x8_t p = {0, 0, 0, 0, 0, 0, 0, 0};
            if (j < a.r) {
                const int gm = min(row0 + r, a.M - 1);
                const u16x8_t v = *(const u16x8_t *)(a.ext_act + (long)gm * a.r + j);
#pragma unroll
                for (int h = 0; h < 8; ++h) p[h] = to16<BF16>(a.sc * cvt16<BF16>(v[h]));
            }
            *(u16x8_t *)(As + r * LDS_STRIDE + j) = p;
        }
        for (int c = tid; c < BN * cpr; c += THREADS) {
            const int r = c / cpr, j = (c % cpr) * 8;
            const int col = col0 + r;
            u16x8_t p = {0, 0, 0, 0, 0, 0, 0, 0};
            if (j < a.r && col < NO) {
                if constexpr (TRANS) {
#pragma unroll
                    for (int h = 0; h < 8; ++h) p[h] = a.ext_w[(long)(j + h) * a.K + col];
                } else {
                    p = *(const u16x8_t *)(a.ext_w + (long)col * a.r + j);
                }
            }
            *(u16x8_t *)(Bs + r * LDS_STRIDE + j) = p;
        }
        __syncthreads();
        for (int ks = 0; ks < nsteps; ++ks) {
            Frags f;
            load_frags(0, ks, f);
            mfma_frags(f);
        }
    }

    // --- epilogue: fp32 accumulators -> 16 bit.  Each wave lays its TM x TN block into its own LDS area in row-major
    //     order, then streams it out in 16-byte pieces (8 lanes per 128-byte row segment).  Rows beyond M and
    //     columns beyond NO (always whole 8-element pieces) are dropped.
    __syncthreads();
    {
        constexpr int ESTR = TN + 8;
        uint16_t *E = smem + wave * (TM * ESTR);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    E[(i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * ESTR + j * 32 + (lane & 31)] =
                        to16<BF16>(acc[i][j][v]);
        __syncthreads();
        constexpr int CPR = TN / 8;                       // 16-byte pieces per row
        const int rbase = row0 + wm * TM, cbase = col0 + wn * TN;
#pragma unroll
        for (int q = 0; q < TM * CPR / 64; ++q) {
            const int c = lane + 64 * q, r = c / CPR, ch = (c % CPR) * 8;
            const u32x4_t v = *(const u32x4_t *)(E + r * ESTR + ch);
            if (rbase + r < a.M && cbase + ch < NO) *(u32x4_t *)(a.out + ((long)(rbase + r) * NO + cbase + ch)) = v;
        }
    }
}

template <int BITS, bool BF16, bool TRANS, int BM, int BN, int WM, int WN>
void launch_variant(const GemmArgs &a, hipStream_t s)
{
    constexpr size_t lds_pipe = 2 * (size_t)(BM + BN) * LDS_STRIDE * sizeof(uint16_t);
    constexpr size_t lds_epi = 4 * (size_t)(BM / WM) * (BN / WN + 8) * sizeof(uint16_t);
    constexpr size_t lds = lds_pipe > lds_epi ? lds_pipe : lds_epi;
    auto kern = qgemm_kernel<BITS, BF16, TRANS, BM, BN, WM, WN>;
    static bool configured = false;   // raising the dynamic-LDS ceiling is a property of the function, set once
    if (!configured) {
        (void)hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        configured = true;
    }
    hipLaunchKernelGGL(kern, dim3(a.tiles_m * a.tiles_n), dim3(THREADS), lds, s, a);
}

template <int BITS, bool BF16, bool TRANS>
void launch_tiles(GemmArgs &a, hipStream_t s)
{
    constexpr int BM = 256, BN = 128;
    const int NO = TRANS ? a.K : a.N;
    a.tiles_m = (a.M + BM - 1) / BM;
    a.tiles_n = (NO + BN - 1) / BN;
    launch_variant<BITS, BF16, TRANS, BM, BN, 2, 2>(a, s);
}

// Multiplier m with umulhi(q, m) == q / (G/32) for every q < 2^16 (q = k/32, K < 2^21): m = floor(2^32 / d) + 1
// for d = G/32 >= 2.  d = 1 would need m = 2^32; it is encoded as 0 and the kernel then uses q itself.
inline uint32_t group_magic(int G)
{
    const uint32_t d = (uint32_t)(G / 32);
    return d == 1 ? 0u : (uint32_t)(0x100000000ull / d) + 1u;
}

template <bool TRANS>
void launch_bits_dtype(const Problem &p, GemmArgs &a, hipStream_t s)
{
#define QLORA_CASE(B)                                   \
    case B:                                             \
        if (p.bf16) launch_tiles<B, true, TRANS>(a, s); \
        else launch_tiles<B, false, TRANS>(a, s);       \
        break
    switch (p.bits) {
        QLORA_CASE(2);
        QLORA_CASE(3);
        QLORA_CASE(4);
    default:
        if (p.bf16) launch_tiles<8, true, TRANS>(a, s);
        else launch_tiles<8, false, TRANS>(a, s);
        break;
    }
#undef QLORA_CASE
}

}  // namespace

void launch_fwd_mfma(const Problem &p, const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                     const void *t, const void *B, void *y, hipStream_t s)
{
    GemmArgs a{(const uint16_t *)x, packed, (const uint16_t *)scales, zeros, (const uint16_t *)t, (const uint16_t *)B,
               (uint16_t *)y, p.M, p.N, p.K, p.G, p.r, p.sc, 0, 0, group_magic(p.G)};
    launch_bits_dtype<false>(p, a, s);
}

void launch_bwd_dx_mfma(const Problem &p, const void *dy, const uint32_t *packed, const void *scales,
                        const uint8_t *zeros, const void *u, const void *A, void *dx, hipStream_t s)
{
    GemmArgs a{(const uint16_t *)dy, packed, (const uint16_t *)scales, zeros, (const uint16_t *)u, (const uint16_t *)A,
               (uint16_t *)dx, p.M, p.N, p.K, p.G, p.r, p.sc, 0, 0, group_magic(p.G)};
    launch_bits_dtype<true>(p, a, s);
}

}  // namespace qlora
