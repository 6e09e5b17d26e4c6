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

// Code i (compile-time) of a 32-code unit held in BITS words.
template <int BITS>
__device__ __forceinline__ uint32_t unit_code(const uint32_t (&w)[BITS], int i)
{
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int o = BITS * i, wi = o >> 5, sh = o & 31;
    uint32_t q = w[wi] >> sh;
    if (sh + BITS > 32) q |= w[wi + 1] << (32 - sh);
    return q & mask;
}

// Dequantise one unit: out[i] = round16(s * (q_i - z)).
template <int BITS, bool BF16>
__device__ __forceinline__ void dequant_unit(const uint32_t (&w)[BITS], float s, float z, uint16_t (&out)[32])
{
#pragma unroll
    for (int i = 0; i < 32; ++i) out[i] = to16<BF16>(((float)unit_code<BITS>(w, i) - z) * s);
}

template <int BITS, bool BF16, bool TRANS, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(THREADS) void qgemm_kernel(const GemmArgs a)
{
    static_assert(WM * WN == 4, "four waves per workgroup");
    static_assert(BN % 128 == 0 && BM % 32 == 0, "tile shape");
    constexpr int TM = BM / WM, TN = BN / WN;       // per-wave output tile
    constexpr int MI = TM / 32, NI = TN / 32;       // 32x32 MFMA blocks per wave
    constexpr int XCH = BM * (BK / 8) / THREADS;    // 16-byte activation chunks per thread per stage
    constexpr int WU = BN / 128;                    // 32-code weight units per thread per stage
    constexpr int STAGE = (BM + BN) * LDS_STRIDE;   // halfs per LDS stage

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

    u32x4_t xr[XCH];
    uint32_t wr[WU][BITS];
    float ws[WU], wz[WU];

    auto load_global = [&](int kt) {
        const int kbase = kt * BK;
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int c = tid + THREADS * i, r = c >> 3, kc = (c & 7) * 8;
            const int gm = min(row0 + r, a.M - 1), k = kbase + kc;
            if (k < KC)
                xr[i] = *(const u32x4_t *)(a.act + (long)gm * KC + k);
            else
                xr[i] = u32x4_t{0u, 0u, 0u, 0u};
        }
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
                n = min(n, a.N - 1);
            }
            if (ok) {
                load_unit<BITS>(a.packed + (long)n * Kw + (k0 >> 5) * BITS, wr[i]);
                const long gi = (long)n * ng + k0 / a.G;
                ws[i] = f16_bits_to_f32(a.scales[gi]);
                wz[i] = (float)a.zeros[gi];
            } else {
#pragma unroll
                for (int j = 0; j < BITS; ++j) wr[i][j] = 0u;
                ws[i] = 0.f;
                wz[i] = 0.f;
            }
        }
    };

    auto store_lds = [&](int buf) {
        uint16_t *As = smem + buf * STAGE, *Bs = As + BM * LDS_STRIDE;
#pragma unroll
        for (int i = 0; i < XCH; ++i) {
            const int c = tid + THREADS * i, r = c >> 3, kc = (c & 7) * 8;
            *(u32x4_t *)(As + r * LDS_STRIDE + kc) = xr[i];
        }
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const int u = tid + THREADS * i;
            uint16_t v[32];
            dequant_unit<BITS, BF16>(wr[i], ws[i], wz[i], v);
            if constexpr (TRANS) {
                const int nl = u & 63, kl = (u >> 6) * 32;
#pragma unroll
                for (int e = 0; e < 32; ++e) Bs[(kl + e) * LDS_STRIDE + nl] = v[e];
            } else {
                uint16_t *dst = Bs + (u >> 1) * LDS_STRIDE + (u & 1) * 32;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    u16x8_t p;
#pragma unroll
                    for (int h = 0; h < 8; ++h) p[h] = v[8 * e + h];
                    *(u16x8_t *)(dst + 8 * e) = p;
                }
            }
        }
    };

    auto compute = [&](int buf, int nsteps) {
        const uint16_t *As = smem + buf * STAGE, *Bs = As + BM * LDS_STRIDE;
        const int fr = lane & 31, fk = (lane >> 5) * 8;
        for (int ks = 0; ks < nsteps; ++ks) {
            u16x8_t af[MI], bf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) af[i] = *(const u16x8_t *)(As + (wm * TM + i * 32 + fr) * LDS_STRIDE + ks * 16 + fk);
#pragma unroll
            for (int j = 0; j < NI; ++j) bf[j] = *(const u16x8_t *)(Bs + (wn * TN + j * 32 + fr) * LDS_STRIDE + ks * 16 + fk);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[i][j] = mfma32<BF16>(af[i], bf[j], acc[i][j]);
        }
    };

    // --- main loop over the contraction, LDS double-buffered, next stage prefetched into registers
    const int KT = (KC + BK - 1) / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        if (kt + 1 < KT) load_global(kt + 1);
        compute(kt & 1, BK / 16);
        if (kt + 1 < KT) store_lds((kt + 1) & 1);
        __syncthreads();
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
        compute(0, nsteps);
    }

    // --- epilogue: fp32 accumulators -> 16 bit, rows beyond M and columns beyond NO are dropped
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int col = col0 + wn * TN + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm * TM + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (row < a.M && col < NO) a.out[(long)row * NO + col] = to16<BF16>(acc[i][j][v]);
            }
        }
}

template <int BITS, bool BF16, bool TRANS, int BM, int BN, int WM, int WN>
void launch_variant(const GemmArgs &a, hipStream_t s)
{
    constexpr size_t lds = 2 * (size_t)(BM + BN) * LDS_STRIDE * sizeof(uint16_t);
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
               (uint16_t *)y, p.M, p.N, p.K, p.G, p.r, p.sc, 0, 0};
    launch_bits_dtype<false>(p, a, s);
}

void launch_bwd_dx_mfma(const Problem &p, const void *dy, const uint32_t *packed, const void *scales,
                        const uint8_t *zeros, const void *u, const void *A, void *dx, hipStream_t s)
{
    GemmArgs a{(const uint16_t *)dy, packed, (const uint16_t *)scales, zeros, (const uint16_t *)u, (const uint16_t *)A,
               (uint16_t *)dx, p.M, p.N, p.K, p.G, p.r, p.sc, 0, 0};
    launch_bits_dtype<true>(p, a, s);
}

}  // namespace qlora
