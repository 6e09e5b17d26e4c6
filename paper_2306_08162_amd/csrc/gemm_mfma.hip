// Tiled MFMA GEMM over the packed weight with dequantisation fused into the operand staging.
//
//   forward   (TRANS = false):  y [M,N]  = x [M,K]  * Wd[N,K]^T  + sc * t[M,r] * B[N,r]^T      (Fig. 1, forward path)
//   backward  (TRANS = true):   dX[M,K]  = dY[M,N]  * Wd[N,K]    + sc * u[M,r] * A[r,K]        (Sec. 3.1: the packed
//             weight is consumed transposed; transpose + unpack + matmul happen inside this one kernel)
//
// Both are C[M,NO] = Act[M,KC] * W^T with W viewed as [NO,KC]; only the way a packed tile is fetched and laid
// into LDS differs.  A workgroup owns a BM x BN output tile and walks the contraction in steps of 64 through a
// double-buffered LDS stage.  Its eight waves are specialised: four staging waves move activation chunks
// global -> registers -> LDS unchanged and packed words global -> registers -> (unpack, s*(q-z), round to 16 bit)
// -> LDS; four MFMA waves read 16-byte fragments from LDS into v_mfma_f32_32x32x16.  One barrier per stage.
// The dequantised weight never reaches HBM.  The rank-r LoRA term is folded in as extra contraction steps.
#include "common.hpp"
#include "dequant.hpp"
#include "kernels.hpp"

namespace qlora {

namespace {

constexpr int BK = 64;               // contraction elements per LDS stage
constexpr int LDS_STRIDE = BK + 8;   // 144-byte rows: the 16-byte reads of 8 consecutive rows fall in distinct bank groups
constexpr int THREADS = 512;        // 4 MFMA waves + 4 staging waves
constexpr int STAGERS = 256;        // staging threads

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
    uint16_t s[WU];     // raw fp16 bits: nothing may touch loaded values before they are staged, or the
    uint8_t z[WU];      // in-order memory counter would make that instruction wait for every load issued so far
    bool ok[WU];        // false: the unit lies outside the weight, stage zeros
};

template <int BITS, bool BF16, bool TRANS, int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(THREADS) void qgemm_kernel(const GemmArgs a)
{
    static_assert(WM * WN == 4, "four MFMA waves per workgroup");
    static_assert(BN % 128 == 0 && BM % 128 == 0, "tile shape");
    constexpr int TM = BM / WM, TN = BN / WN;       // per-wave output tile
    constexpr int MI = TM / 32, NI = TN / 32;       // 32x32 MFMA blocks per wave
    constexpr int XCH = BM * (BK / 8) / STAGERS;    // 16-byte activation chunks per staging thread per stage
    constexpr int WU = BN / 128;                    // 32-code weight units per staging thread per stage
    constexpr int STAGE = (BM + BN) * LDS_STRIDE;   // halfs per LDS stage
    constexpr int KSTEPS = BK / 16;                 // MFMA k-steps per stage
    using Regs = StageRegs<BITS, XCH, WU>;

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];

    // Waves 0-3 only feed the matrix cores (LDS fragment reads + MFMA); waves 4-7 only stage operands (global
    // loads, dequantisation, LDS writes).  Each SIMD hosts one wave of each kind, so the vector ALU work of the
    // dequantisation issues in the shadow of the other wave's MFMAs instead of competing for its issue slots.
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool stager = wave >= 4;
    const int stid = tid & (STAGERS - 1);           // index among the staging threads
    const int cw = wave & 3, wm = cw / WN, wn = cw % WN;
    const int NO = TRANS ? a.K : a.N;    // output columns
    const int KC = TRANS ? a.N : a.K;    // contraction length
    const int ng = a.K / a.G, Kw = a.K * BITS / 32;
    const int KT = (KC + BK - 1) / BK;

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
    // One k-step of the MFMA waves: the fragments of a later k-step are requested from LDS while the MFMAs of the
    // current one issue, one LDS read slotted behind each MFMA so the matrix pipe never waits on a burst of reads.
    auto kstep = [&](int rbuf, int rks, Frags &into, const Frags &use) {
#ifndef QLORA_EXP_NOFRAG
        load_frags(rbuf, rks, into);
#endif
        mfma_frags(use);
#pragma unroll
        for (int i = 0; i < MI * NI; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA
            if (i < MI + NI) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);       // one LDS read
        }
    };

    if (stager) {
        // global -> registers for stage kt.  Branch-free: every address is clamped into the valid range and
        // whatever lies beyond the contraction length (or beyond the weight's rows / columns) is neutralised by a
        // zero scale on the weight side, so stages past the end may be fetched and staged harmlessly.
        const uint32_t xkc = (stid & 7) * 8;                // same k offset for every chunk of this thread
        uint32_t xrow_off[XCH];                             // element offset of each chunk's row
#pragma unroll
        for (int i = 0; i < XCH; ++i)
            xrow_off[i] = (uint32_t)min(row0 + ((stid + STAGERS * i) >> 3), a.M - 1) * (uint32_t)KC;

#ifndef QLORA_PHASE_MODE
#define QLORA_PHASE_MODE 0
#endif
        const int phase = QLORA_PHASE_MODE == 0 ? 0
                          : QLORA_PHASE_MODE == 1 ? (pm * KT) / a.tiles_m
                          : QLORA_PHASE_MODE == 2 ? ((pm * KT) / a.tiles_m + pn) % KT
                                                  : (pn * 5 + pm * 3) % KT;
        auto load_global = [&](int kt_seq, Regs &rg) {
            int kt = kt_seq + phase;
            kt = kt >= KT ? kt - KT : kt;               // stages are visited in a rotated order (see above)
            const int kbase = kt * BK;
            const uint32_t k = (uint32_t)min(kbase + (int)xkc, KC - 8);
#pragma unroll
            for (int i = 0; i < XCH; ++i) rg.x[i] = *(const u32x4_t *)(a.act + (xrow_off[i] + k));
#pragma unroll
            for (int i = 0; i < WU; ++i) {
                const int u = stid + STAGERS * i;
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
#ifdef QLORA_EXP_NOWLOAD
                for (int j = 0; j < BITS; ++j) rg.w[i][j] = 0x12345678u + n;
#else
                load_unit<BITS>(a.packed + (long)n * Kw + (k0 >> 5) * BITS, rg.w[i]);
#endif
                const long gi = (long)n * ng + (a.g32_magic ? (int)__umulhi((uint32_t)(k0 >> 5), a.g32_magic) : (k0 >> 5));
#ifdef QLORA_EXP_NOSZLOAD
                rg.s[i] = (uint16_t)gi;
                rg.z[i] = (uint8_t)gi;
#else
                rg.s[i] = a.scales[gi];
                rg.z[i] = a.zeros[gi];
#endif
                rg.ok[i] = ok;
            }
        };

        // registers -> LDS: activation chunks unchanged, every unit dequantised 8 codes at a time
        auto stage = [&](const Regs &rg, int buf) {
            uint16_t *As = smem + buf * STAGE, *Bs = As + BM * LDS_STRIDE;
#ifdef QLORA_EXP_NOXW
            {
                u32x4_t t = rg.x[0];
                for (int i = 1; i < XCH; ++i) t ^= rg.x[i];
                if (t[0] == 0x12345678u) *(u32x4_t *)(As + stid * 8) = t;
            }
#else
#pragma unroll
            for (int i = 0; i < XCH; ++i) {
                const int c = stid + STAGERS * i, r = c >> 3, kc = (c & 7) * 8;
                *(u32x4_t *)(As + r * LDS_STRIDE + kc) = rg.x[i];
            }
#endif
#ifdef QLORA_EXP_NOWW
            if (rg.w[0][0] == 0x12345678u && rg.s[0] == 77 && rg.z[0] == 3) Bs[stid] = 1;
            return;
#endif
#pragma unroll
            for (int i = 0; i < WU; ++i) {
                const int u = stid + STAGERS * i;
                DequantConst<BITS, BF16> dq;
                dq.set(rg.ok[i] ? f16_bits_to_f32(rg.s[i]) : 0.f, (float)rg.z[i]);
#pragma unroll
                for (int part = 0; part < 4; ++part) {
#ifdef QLORA_EXP_NODEQ
                    u16x8_t v;
                    for (int e = 0; e < 8; ++e) v[e] = (uint16_t)(rg.w[i][0] + e);
#else
                    const u16x8_t v = dequant8<BITS, BF16>(rg.w[i], part, dq);
#endif
                    if constexpr (TRANS) {
                        uint16_t *dst = Bs + ((u >> 6) * 32 + part * 8) * LDS_STRIDE + (u & 63);
#pragma unroll
                        for (int e = 0; e < 8; ++e) dst[e * LDS_STRIDE] = v[e];
                    } else {
                        *(u16x8_t *)(Bs + (u >> 1) * LDS_STRIDE + (u & 1) * 32 + part * 8) = v;
                    }
                }
            }
        };

        // stage kt+1 is written while the MFMA waves work on stage kt; NSETS later stages are in flight from
        // memory (one register set each), enough to cover the L2 / HBM round trip with a full stream of loads
        constexpr int NSETS = 3;
        Regs rs[NSETS];
#pragma unroll
        for (int i = 0; i < NSETS; ++i) load_global(i, rs[i]);
        stage(rs[0], 0);
        load_global(NSETS, rs[0]);
        __syncthreads();
        // One step: the MFMA waves work on stage kt while stage kt+1 (held in set (i+1) % NSETS) goes to LDS and
        // that set is refilled with stage kt+1+NSETS.
        auto step = [&](int kt, Regs &rg) {
#ifndef QLORA_EXP_NOSTAGE
            stage(rg, (kt + 1) & 1);
#endif
#ifndef QLORA_EXP_NOLOAD
            load_global(kt + 1 + NSETS, rg);
#endif
#ifndef QLORA_EXP_NOBAR
            __syncthreads();
#endif
        };
        // Whole rotations run without any condition inside: the compiler derives how many loads may stay in flight
        // from the static paths through the loop, and a skippable step would make it assume the shortest one.
        int kt0 = 0;
        for (; kt0 + NSETS <= KT; kt0 += NSETS) {
#pragma unroll
            for (int i = 0; i < NSETS; ++i) step(kt0 + i, rs[(i + 1) % NSETS]);
        }
#pragma unroll
        for (int i = 0; i < NSETS - 1; ++i)
            if (kt0 + i < KT) step(kt0 + i, rs[(i + 1) % NSETS]);
    } else {
        // MFMA waves.  The last k-step of a stage runs from registers after the barrier, overlapping the LDS
        // latency of the next stage's first fragments.
        Frags f[2];
        __syncthreads();
        load_frags(0, 0, f[0]);
        for (int kt = 0; kt < KT; ++kt) {
            const int buf = kt & 1;
#ifndef QLORA_EXP_NOMFMA
            kstep(buf, 1, f[1], f[0]);
            kstep(buf, 2, f[0], f[1]);
            kstep(buf, 3, f[1], f[0]);
#ifndef QLORA_EXP_NOBAR
            __syncthreads();
#endif
            kstep(buf ^ 1, 0, f[0], f[1]);
#else
            __syncthreads();
#endif
        }
    }

    // --- LoRA term as extra contraction steps: Act' = sc * t (or u), W' = B (or A^T), zero-padded to 16.
    //     Every wave is past the last barrier of the main loop, so both LDS stages are free.
    if (a.r > 0) {
        const int nsteps = (a.r + 15) / 16, width = nsteps * 16;
        if (stager) {
            uint16_t *As = smem, *Bs = As + BM * LDS_STRIDE;
            const int cpr = width / 8;                      // 8-element chunks per row
            for (int c = stid; c < BM * cpr; c += STAGERS) {
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
            for (int c = stid; c < BN * cpr; c += STAGERS) {
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
        }
        __syncthreads();
        if (!stager) {
            for (int ks = 0; ks < nsteps; ++ks) {
                Frags fx;
                load_frags(0, ks, fx);
                mfma_frags(fx);
            }
        }
        __syncthreads();
    }

    // --- epilogue: fp32 accumulators -> 16 bit.  Each MFMA wave lays its TM x TN block into its own LDS area in
    //     row-major order; then all eight waves stream the areas out in 16-byte pieces (8 lanes per 128-byte row
    //     segment).  Rows beyond M and columns beyond NO (always whole 8-element pieces) are dropped.
    constexpr int ESTR = TN + 8;
    if (!stager) {
        uint16_t *E = smem + cw * (TM * ESTR);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    E[(i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * ESTR + j * 32 + (lane & 31)] =
                        to16<BF16>(acc[i][j][v]);
    }
    __syncthreads();
    {
        constexpr int CPR = TN / 8;                       // 16-byte pieces per row of one wave's area
        constexpr int PER_AREA = TM * CPR;
#pragma unroll
        for (int q = 0; q < 4 * PER_AREA / THREADS; ++q) {
            const int c = tid + THREADS * q, w = c / PER_AREA, cc = c % PER_AREA;
            const int r = cc / CPR, ch = (cc % CPR) * 8;
            const int grow = row0 + (w / WN) * TM + r, gcol = col0 + (w % WN) * TN + ch;
            const u32x4_t v = *(const u32x4_t *)(smem + w * (TM * ESTR) + r * ESTR + ch);
            if (grow < a.M && gcol < NO) *(u32x4_t *)(a.out + ((long)grow * NO + gcol)) = v;
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
#ifndef QLORA_BM
#define QLORA_BM 256
#define QLORA_BN 128
#endif
    constexpr int BM = QLORA_BM, BN = QLORA_BN;
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
