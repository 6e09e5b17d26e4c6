// Tiled MFMA GEMM over the packed weight with dequantisation fused into the operand staging.
//
//   forward   (TRANS = false):  y [M,N]  = x [M,K]  * Wd[N,K]^T  + sc * t[M,r] * B[N,r]^T      (Fig. 1, forward path)
//   backward  (TRANS = true):   dX[M,K]  = dY[M,N]  * Wd[N,K]    + sc * u[M,r] * A[r,K]        (Sec. 3.1: the packed
//             weight is consumed transposed; transpose + unpack + matmul happen inside this one kernel)
//
// Both are C[M,NO] = Act[M,KC] * W^T with W viewed as [NO,KC]; only the way a packed tile is fetched and laid
// into LDS differs.  A workgroup owns a BM x BN output tile and walks the contraction in steps of 64.  Its eight
// waves are specialised: four staging waves move packed words global -> registers -> (unpack, s*(q-z), round to
// 16 bit) -> LDS (two stages); four MFMA waves pull the activation tile global -> LDS directly (three stages, no
// registers) and read 16-byte fragments of both operands into v_mfma_f32_32x32x16.  One barrier per stage.
// The dequantised weight never reaches HBM.  The rank-r LoRA term is folded in as extra contraction steps.
// Launches that give every compute unit at least one 256 x 256 tile use a second arrangement of the same parts
// (SYM below): eight waves that each stage, load and multiply an eighth.
#include "common.hpp"
#include "dequant.hpp"
#include "kernels.hpp"

namespace qlora {

namespace {

constexpr int BK = 64;               // contraction elements per LDS stage
constexpr int GEMM_NXS = 3;     // activation stages in LDS
constexpr int LDS_STRIDE = BK + 8;   // 144-byte rows: the 16-byte reads of 8 consecutive rows fall in distinct bank groups
constexpr int STAGERS = 256;        // staging threads (4 waves); the MFMA waves come on top

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
    float *part;              // splits > 1: fp32 partial products [splits][M][NO], summed by splitk_sum_kernel
    int splits, kt_split;     // workgroups per tile along the contraction, 64-deep stages per workgroup
    const uint8_t *keep;      // LoRA dropout (backward only): keep bit of x[m, k] is bit k % 8 of keep[m * K/8 + k/8]
    float keep_sc;            // sc * keep_scale
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

// What one staging thread fetches for one 64-deep stage of the weight: WU packed units with their group's scale
// and zero-point, kept exactly as loaded.
template <int BITS, int WU>
struct StageRegs {
    uint32_t w[WU][BITS];
    uint16_t s[WU];     // raw fp16 bits: nothing may touch loaded values before they are staged, or the
    uint8_t z[WU];      // in-order memory counter would make that instruction wait for every load issued so far
    bool ok[WU];        // false: the unit lies outside the weight, stage zeros
};

// wait until at most N vector-memory operations of this wave are outstanding, then meet the workgroup
template <int N>
__device__ __forceinline__ void wait_vm_and_barrier()
{
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Swizzle key of a row of the backward weight stage.  Its upper two bits run through 0..3 over any 4 consecutive
// rows starting at a multiple of 4 (the transposing reads), its lower three bits through 0..7 over any 8 consecutive
// rows starting at a multiple of 8 (the 16-byte writes, one row per lane: eight lanes per clock into a bank space of
// 128 bytes.  Counters: with a key whose lower three bits took four values, a write took 16 LDS cycles instead of 8).
__device__ __forceinline__ constexpr int wswz(int row) { return ((row & 3) << 2) | (row & 2) | ((row >> 2) & 1); }
// Slot key of a row of the forward weight stage of the symmetric arrangement (128-byte rows): eight different values
// over the even and over the odd rows of any 16 consecutive rows (16-byte reads: sixteen lanes per clock, two rows
// fill the 256-byte bank space), four different values mod 4 over any 4 consecutive rows (16-byte writes: two
// lanes per row, pieces p and p + 4, eight lanes per clock into 128 bytes).
__device__ __forceinline__ constexpr int fswz(int row) { return ((row & 3) ^ ((row >> 2) & 1)) | (((row >> 3) & 1) << 2); }

// MASKED (backward under LoRA dropout, ranks up to 32, no split): the adapter's share of dX is masked per element,
// dX = dY Wd + keep_sc * keep (.) (u A), so it cannot ride in the accumulators.  The LoRA steps are left out; the
// staging waves lay the tile's rows of u and columns of A (both fetched at kernel start) beside the epilogue area, and
// the copy-out adds the masked product to every 8-element piece before it is stored.
//
// SYM (256 x 256 tiles, for launches of at least one such tile per compute unit): four waves, one per SIMD, each with
// a 128 x 128 block of accumulators (256 registers, which leaves no room for a second wave on the SIMD) and each
// doing a quarter of everything: activation loads, weight staging and the MFMAs.  Twice the flops per byte moved
// through LDS and through the direct-to-LDS path of the 256 x 128 tile.
template <int BITS, bool BF16, bool TRANS, int BM, int BN, int WM, int WN, bool MASKED = false, bool SYM = false>
__global__ __launch_bounds__(WM * WN * 64 + (SYM ? 0 : STAGERS)) void qgemm_kernel(const GemmArgs a)
{
    static_assert(!MASKED || TRANS, "the dropout mask acts on dX only");
    constexpr int MW = WM * WN;                     // MFMA waves
    constexpr int THREADS = MW * 64 + (SYM ? 0 : STAGERS);
    static_assert(MW == 4 || MW == 8, "one or two MFMA waves per SIMD");
    static_assert(!SYM || !MASKED, "symmetric waves: no masked epilogue");
    constexpr int NSTG = SYM ? MW * 64 : STAGERS;   // staging threads: all of them, or the four staging waves
    static_assert(BN % 128 == 0 && BM % 128 == 0, "tile shape");
    constexpr int TM = BM / WM, TN = BN / WN;       // per-wave output tile
    constexpr int MI = TM / 32, NI = TN / 32;       // 32x32 MFMA blocks per wave
    constexpr int XDMA = BM / 8 / MW;               // direct-to-LDS loads per MFMA wave per stage (8 rows each)
    static_assert(XDMA >= 4 && XDMA % 4 == 0, "loads are spread over the four k-steps");
    constexpr int WU = 2 * BN / NSTG;               // 32-code weight units per staging thread per stage
    constexpr int XS = BM * BK;                     // halfs per activation stage (128-byte rows, swizzled)
    constexpr int NXS = GEMM_NXS;                   // (2 would let two workgroups share a CU's LDS: measured slower)
    static_assert(NXS == 2 || NXS == 3, "activation stages");
    // Weight stage.  Forward: [BN rows n][64 k + 8] (144-byte rows), fragments are 16-byte reads.  Backward: the
    // staging threads own rows n of the contraction, so the stage is kept as they produce it, [64 rows n][BN k],
    // and the fragments are gathered with the transposing LDS read (ds_read_b64_tr_b16), two per fragment.  The
    // 16-byte pieces of a row are XOR-swizzled with wswz(row): eight consecutive rows put the same piece into
    // eight different bank quads of the 128 bytes a write cycle covers (the stagers' 16-byte writes, one row per
    // lane), and four consecutive rows put four consecutive pieces into disjoint runs of 16 banks (the transposing
    // reads: 4 rows x 64 bytes per half wave).  Unpadded 320-byte rows served the reads equally well but made the
    // writes collide four ways.
    // SYM, forward: 128-byte rows with a slot swizzle (fswz) instead of the padding (LDS is full).
    constexpr int WPITCH = TRANS ? BN : (SYM ? BK : LDS_STRIDE);
    constexpr int WS = TRANS ? BK * WPITCH : BN * WPITCH;       // halfs per weight stage
    using Regs = StageRegs<BITS, WU>;

    extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
    uint16_t *const xs = smem;                      // [NXS][BM][64]
    uint16_t *const wsm = smem + NXS * XS;          // [2] weight stages

    // The first MW waves feed the matrix cores: LDS fragment reads, MFMAs, and the direct-to-LDS loads of the
    // activation tile (no registers, no ALU work).  The last four waves stage the weight: packed words global ->
    // registers -> dequantise -> LDS.  Every SIMD hosts waves of both kinds (and, with MW = 8, two MFMA waves), so
    // one wave's fragment reads, loads and dequantisation issue in the shadow of another wave's MFMAs: a single
    // wave cannot hide its own instruction issue behind its MFMAs.
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, kept in a scalar register
    const bool stager = SYM || wave >= MW, feeder = SYM || wave < MW;
    const int stid = SYM ? tid : tid - MW * 64;     // index among the staging threads
    const int cw = wave, wm = cw / WN, wn = cw % WN;
    const int NO = TRANS ? a.K : a.N;    // output columns
    const int KC = TRANS ? a.N : a.K;    // contraction length
    const int ng = a.K / a.G, Kw = a.K * BITS / 32;
    // a workgroup owns the stages kt_first .. kt_first + KT of its tile's contraction (all of them unless the
    // contraction is split over several workgroups)
    const int nt = a.tiles_m * a.tiles_n;
    const int split = __builtin_amdgcn_readfirstlane(a.splits > 1 ? (int)blockIdx.x / nt : 0);
    const int kt_first = split * a.kt_split;
    const int KT = min((KC + BK - 1) / BK - kt_first, a.kt_split);

    // --- which tile: consecutive workgroups land on different XCDs, so hand each XCD a contiguous run of tile
    //     ids, and order ids so that a run covers a compact block of tiles (shared rows and columns hit in L2)
    int pm, pn;
    {
        const int bid = a.splits > 1 ? (int)blockIdx.x % nt : (int)blockIdx.x;
        const int xcd = bid & 7, loc = bid >> 3, per = nt >> 3, rem = nt & 7;
        const int t = xcd * per + min(xcd, rem) + loc;
        // Tile ids run down GM tile rows before they move to the next tile column.  An activation tile row is 32 / bits
        // times the bytes of a packed weight tile column, so a run should be wide rather than tall: with 32 tiles per
        // XCD (the headline launch) GM = 2 makes it 2 x 16 and the launch fetches 69 MB where GM = 4 (4 x 8) fetched
        // 85 MB; the time is the same (the fetches are not what the kernel waits for).
        constexpr int GM = 2;
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

    // Activation tile in LDS: row r is 128 bytes = eight 16-byte slots; slot s holds the row's chunk
    // s ^ ((r >> 1) & 7).  A 16-byte LDS read serves 16 lanes per clock out of a 256-byte-wide bank space, i.e. two
    // rows; with this key the 16 consecutive rows read by 16 lanes fall into 16 different slots of that space.
    // A direct-to-LDS load lays the 64 lanes' 16 bytes down contiguously (8 rows), so the swizzle is applied by
    // choosing which global chunk each lane fetches.
    struct Frags {
        u16x8_t a[MI], b[NI];
    };
    const int fr = lane & 31, fh = lane >> 5;
    int aoff[BK / 16];                              // per k-step: this lane's offset into an activation stage
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) aoff[ks] = (wm * TM + fr) * BK + ((2 * ks + fh) ^ ((fr >> 1) & 7)) * 8;
    // and into a weight stage (a k-step adds 16 contraction elements).  Transposing read: in every block of 16
    // lanes, lane 4e+g supplies the address of four consecutive 16-bit columns of one row, and lane i receives, as
    // element e, column i%4 of the row supplied by lane 4e + i/4.  Lane (e, g) of block b therefore points at row
    // 8 (b/2) + e, columns 16 (b%2) + 4g .. +4 of the 16 x 32 k-step slab, and lane l ends up with contraction
    // elements 8 (l/32) .. +4 of column l % 32: half an MFMA operand; the second read starts four rows further down.
    // The row's swizzle key is 4 e + 2 (l/32) + (second read), so each of the 2 NI reads has its own offset.
    const int boff = TRANS ? 0 : (wn * TN + fr) * WPITCH + (SYM ? 0 : fh * 8);
    int toff[TRANS ? NI : 1][2];
    if constexpr (TRANS) {
        const int e = (lane & 15) >> 2, row = 8 * (lane >> 5) + e;
        const int piece = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);     // 16-byte piece within the 64-byte run
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int hi = 0; hi < 2; ++hi)
                toff[j][hi] = (row + 4 * hi) * WPITCH
                            + (((wn * TN / 8 + 4 * j + piece) ^ wswz(row + 4 * hi)) * 8) + 4 * (lane & 1);
    }
    auto load_frags = [&](int xstage, int wstage, int ks, Frags &f) {
        const uint16_t *As = xs + xstage * XS + aoff[ks];
#pragma unroll
        for (int i = 0; i < MI; ++i) f.a[i] = *(const u16x8_t *)(As + i * 32 * BK);
        if constexpr (TRANS) {
            const uint16_t *Bs = wsm + wstage * WS + ks * 16 * WPITCH;   // 16 rows further: same swizzle keys
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                typedef short s16x4_t __attribute__((ext_vector_type(4)));
                typedef __attribute__((address_space(3))) s16x4_t *lds4_t;
                const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(Bs + toff[j][0]));
                const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds4_t)(Bs + toff[j][1]));
                f.b[j] = u16x8_t{(uint16_t)lo[0], (uint16_t)lo[1], (uint16_t)lo[2], (uint16_t)lo[3],
                                 (uint16_t)hi[0], (uint16_t)hi[1], (uint16_t)hi[2], (uint16_t)hi[3]};
            }
        } else {
            // (SYM: the slot key depends on the row's lower four bits: the same 32 rows further down)
            const uint16_t *Bs = wsm + wstage * WS + boff + (SYM ? ((2 * ks + fh) ^ fswz(fr)) * 8 : ks * 16);
#pragma unroll
            for (int j = 0; j < NI; ++j) f.b[j] = *(const u16x8_t *)(Bs + j * 32 * WPITCH);
        }
    };
    auto mfma_frags = [&](const Frags &f) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) acc[i][j] = mfma32<BF16>(f.a[i], f.b[j], acc[i][j]);
    };

    constexpr int EXT_STEPS = 2;                                        // LoRA steps whose operands are prefetched
    constexpr int EXT_A = BM * 2 / NSTG, EXT_W = BN * 2 / NSTG;   // pieces per staging thread and LoRA step
    u16x8_t ext_a[EXT_STEPS][EXT_A], ext_w[EXT_STEPS][EXT_W];

    // global -> registers for stage kt.  Branch-free: every address is clamped into the valid range and
    // whatever lies beyond the contraction length (or beyond the weight's rows / columns) is neutralised by a
    // zero scale, so stages past the end may be fetched and staged harmlessly.
    auto load_global = [&](int kt, Regs &rg) {
        const int kbase = (kt_first + kt) * BK;
#pragma unroll
        for (int i = 0; i < WU; ++i) {
            const int u = stid + NSTG * i;
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
            rg.s[i] = a.scales[gi];
            rg.z[i] = a.zeros[gi];
            rg.ok[i] = ok;
        }
    };

    // registers -> LDS: every unit dequantised 8 codes at a time; parts p0 .. p1 of unit i
    auto stage_parts = [&](const Regs &rg, int buf, int i, int p0, int p1) {
        uint16_t *Bs = wsm + buf * WS;
        const int u = stid + NSTG * i;
        DequantConst<BITS, BF16> dq;
        dq.set(rg.ok[i] ? f16_bits_to_f32(rg.s[i]) : 0.f, (float)rg.z[i]);
#pragma unroll
        for (int part = p0; part < p1; ++part) {
            const u16x8_t v = dequant8<BITS, BF16>(rg.w[i], part, dq);
            if constexpr (TRANS) {
                *(u16x8_t *)(Bs + (u & 63) * WPITCH + ((((u >> 6) * 4 + part) ^ wswz(u & 63)) * 8)) = v;
            } else if constexpr (SYM) {        // row u / 2, pieces 4 (u % 2) + part
                *(u16x8_t *)(Bs + (u >> 1) * WPITCH + ((((u & 1) * 4 + part) ^ fswz(u >> 1)) * 8)) = v;
            } else {
                *(u16x8_t *)(Bs + (u >> 1) * LDS_STRIDE + (u & 1) * 32 + part * 8) = v;
            }
        }
    };
    auto stage = [&](const Regs &rg, int buf) {
#pragma unroll
        for (int i = 0; i < WU; ++i) stage_parts(rg, buf, i, 0, 4);
    };

    if constexpr (SYM) {
        // ---- symmetric waves: every wave requests an MW-th of the activation tile, stages an MW-th of the weight
        //      stage and multiplies its own block.  Per 64-deep stage and wave: four k-steps of MI NI MFMAs, XDMA
        //      direct-to-LDS requests (a quarter per k-step), WU units dequantised into the other weight buffer (a
        //      quarter of them per k-step) and WU units requested from memory NSETS stages ahead.
        static_assert((WU == 1 || WU == 2) && NXS == 3, "a quarter of the staging per k-step; three activation stages");
        const int drow = lane >> 3;
        const int dchunk = ((lane & 7) ^ ((4 * cw + (drow >> 1)) & 7)) * 8;
        const uint32_t xs_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)xs;
        uint32_t xoff[XDMA];
#pragma unroll
        for (int i = 0; i < XDMA; ++i)
            xoff[i] = (uint32_t)min(row0 + (MW * i + cw) * 8 + drow, a.M - 1) * (uint32_t)KC * 2u;
        auto issue_x = [&](int kt, int stage, int i) {
            const uint32_t k2 = (uint32_t)min((kt_first + kt) * BK + dchunk, KC - 8) * 2u;
            const uint32_t dst = xs_lds + (uint32_t)(stage * XS + (MW * i + cw) * 512) * 2u;
            dma16(a.act, xoff[i] + k2, (uint32_t)__builtin_amdgcn_readfirstlane((int)dst));
        };
        // a k-step's MFMAs with the next fragments' LDS reads slotted between them (the dequantisation and its LDS
        // writes are left to the compiler's own schedule: a hint that placed them too took minutes to compile)
        auto spread = [&]() {
#pragma unroll
            for (int i = 0; i < MI * NI; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA
                if (i < MI + (TRANS ? 2 * NI : NI)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
            }
        };
        // Requests complete in the order they were made.  Per stage a wave first requests its weight units (at least
        // WL instructions), then the XDMA activation pieces for the stage after next; "the activation pieces of the
        // next stage have landed" is therefore "at most XDMA + WL requests are outstanding".
        constexpr int WL = WU * (BITS == 3 ? 3 : (BITS == 8 ? 2 : 1));
        constexpr int NSETS = 3;
        Regs rs[NSETS];
#pragma unroll
        for (int i = 0; i < NSETS; ++i) load_global(i, rs[i]);
#pragma unroll
        for (int i = 0; i < XDMA; ++i) issue_x(0, 0, i);
#pragma unroll
        for (int i = 0; i < XDMA; ++i) issue_x(1, 1, i);
        stage(rs[0], 0);
        load_global(NSETS, rs[0]);
        wait_vm_and_barrier<XDMA + WL>();       // activation stage 0 and every wave's share of weight stage 0 are in LDS
        Frags f[2];
        load_frags(0, 0, 0, f[0]);
        int xstage = 0;
        // stage kt: rg holds the units of stage kt + 1, and is refilled with those of stage kt + 1 + NSETS
        auto step = [&](int kt, Regs &rg) {
            const int wstage = kt & 1, wfill = wstage ^ 1;
            const int xnext = xstage + 1 == NXS ? 0 : xstage + 1;
            const int xfill = xnext + 1 == NXS ? 0 : xnext + 1;
            auto issue_quarter = [&](int qtr) {
#pragma unroll
                for (int i = qtr * (XDMA / 4); i < (qtr + 1) * (XDMA / 4); ++i) issue_x(kt + 2, xfill, i);
            };
            auto stage_quarter = [&](int qtr) {      // WU parts: quarter 4 i / WU + .. of unit i
                stage_parts(rg, wfill, qtr * WU / 4, (qtr * WU) % 4, (qtr * WU) % 4 + WU);
            };
            load_frags(xstage, wstage, 1, f[1]);
            stage_quarter(0);
            mfma_frags(f[0]);
            spread();
            issue_quarter(0);
            load_frags(xstage, wstage, 2, f[0]);
            stage_quarter(1);
            mfma_frags(f[1]);
            spread();
            issue_quarter(1);
            load_frags(xstage, wstage, 3, f[1]);
            stage_quarter(2);
            mfma_frags(f[0]);
            spread();
            issue_quarter(2);
            stage_quarter(3);
            issue_quarter(3);
            wait_vm_and_barrier<XDMA + WL>();   // activation stage kt + 1 has landed; weight stage kt + 1 is written
            load_global(kt + 1 + NSETS, rg);
            load_frags(xnext, wfill, 0, f[0]);
            mfma_frags(f[1]);
            spread();
            xstage = xnext;
        };
        int kt0 = 0;
        for (; kt0 + NSETS <= KT; kt0 += NSETS) {
#pragma unroll
            for (int i = 0; i < NSETS; ++i) step(kt0 + i, rs[(i + 1) % NSETS]);
        }
#pragma unroll
        for (int i = 0; i < NSETS - 1; ++i)
            if (kt0 + i < KT) step(kt0 + i, rs[(i + 1) % NSETS]);
        wait_vm_and_barrier<0>();               // nothing in flight any more: LDS is quiet
    } else
    if (!stager) {
        // ---- MFMA waves ----
        __builtin_amdgcn_s_setprio(1);          // when both kinds of wave are ready, the matrix pipe's feeder goes first
        // direct-to-LDS loads: this wave's load i covers tile rows (MW i + cw) * 8 .. + 8
        const int drow = lane >> 3;              // row within the 8-row block; block b starts at tile row 8 b
        const int dchunk = ((lane & 7) ^ ((4 * cw + (drow >> 1)) & 7)) * 8;   // MW * i * 4 is a multiple of 8
        const uint32_t xs_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint16_t *)xs;
        uint32_t xoff[XDMA];                    // byte offset of this lane's row within the activation matrix
#pragma unroll
        for (int i = 0; i < XDMA; ++i)
            xoff[i] = (uint32_t)min(row0 + (MW * i + cw) * 8 + drow, a.M - 1) * (uint32_t)KC * 2u;
        auto issue_x = [&](int kt, int stage, int i) {
            // stages past the end and chunks past the contraction length re-read valid data; the weight side is zero there
            const uint32_t k2 = (uint32_t)min((kt_first + kt) * BK + dchunk, KC - 8) * 2u;
            const uint32_t dst = xs_lds + (uint32_t)(stage * XS + (MW * i + cw) * 512) * 2u;   // wave-uniform byte address
            dma16(a.act, xoff[i] + k2, (uint32_t)__builtin_amdgcn_readfirstlane((int)dst));
        };
        // One k-step: the fragments of a later k-step are requested from LDS while the MFMAs of the current one
        // issue, one LDS read slotted behind each MFMA so the matrix pipe never waits on a burst of reads.
        auto kstep = [&](int xstage, int wstage, int rks, Frags &into, const Frags &use) {
            load_frags(xstage, wstage, rks, into);
            mfma_frags(use);
#pragma unroll
            for (int i = 0; i < MI * NI; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                        // one MFMA
                if (i < MI + (TRANS ? 2 * NI : NI)) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
            }
        };

#pragma unroll
        for (int i = 0; i < XDMA; ++i) issue_x(0, 0, i);
        if constexpr (NXS == 3) {
#pragma unroll
            for (int i = 0; i < XDMA; ++i) issue_x(1, 1, i);
        }
        constexpr int AHEAD = NXS == 3 ? XDMA : 0;   // loads that may still be in flight when a stage is needed
        wait_vm_and_barrier<AHEAD>();           // stage 0 of the activations has landed; weights staged by waves 4-7
        Frags f[2];
        load_frags(0, 0, 0, f[0]);
        int xstage = 0;                         // kt % NXS
        for (int kt = 0; kt < KT; ++kt) {
            const int wstage = kt & 1;
            const int xnext = xstage + 1 == NXS ? 0 : xstage + 1;
            const int xfill = NXS == 3 ? (xnext + 1 == NXS ? 0 : xnext + 1) : xnext;   // the stage NXS-1 ahead
            // the last k-step of a stage runs from registers after the barrier, overlapping the LDS latency of the
            // next stage's first fragments; the activation loads for stage kt+2 are spread over the k-steps
            auto issue_quarter = [&](int qtr) {
#pragma unroll
                for (int i = qtr * (XDMA / 4); i < (qtr + 1) * (XDMA / 4); ++i) issue_x(kt + NXS - 1, xfill, i);
            };
            issue_quarter(0);
            kstep(xstage, wstage, 1, f[1], f[0]);
            issue_quarter(1);
            kstep(xstage, wstage, 2, f[0], f[1]);
            issue_quarter(2);
            kstep(xstage, wstage, 3, f[1], f[0]);
            issue_quarter(3);
            wait_vm_and_barrier<AHEAD>();       // stage kt+1 has landed (only loads for a later stage may be pending)
            kstep(xnext, wstage ^ 1, 0, f[0], f[1]);
            xstage = xnext;
        }
        wait_vm_and_barrier<0>();               // the loads issued past the last stage have landed: LDS is quiet
    } else {
        // ---- weight staging waves ----
        // The operands of the LoRA steps that follow the main loop (up to two steps, ranks up to 32) are requested
        // now, so their memory latency is long gone when they are needed: 8-element pieces of t (or u) and of B (or A);
        // piece (row, half h) of step st holds adapter columns 16 st + 8 h .. + 8.
        const int ext_steps = (a.r + 15) / 16;
        if (a.r > 0 && split == 0 && ext_steps <= EXT_STEPS) {
#pragma unroll
            for (int st = 0; st < EXT_STEPS; ++st) {
#pragma unroll
                for (int i = 0; i < EXT_A; ++i) {
                    const int c = stid + NSTG * i, r = c >> 1, j = 16 * st + (c & 1) * 8;
                    ext_a[st][i] = u16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                    if (j < a.r) ext_a[st][i] = *(const u16x8_t *)(a.ext_act + (long)min(row0 + r, a.M - 1) * a.r + j);
                }
#pragma unroll
                for (int i = 0; i < EXT_W; ++i) {
                    const int c = stid + NSTG * i;
                    ext_w[st][i] = u16x8_t{0, 0, 0, 0, 0, 0, 0, 0};
                    if constexpr (TRANS) {
                        const int j = 16 * st + c / (BN / 8), col = col0 + (c % (BN / 8)) * 8;
                        if (j < a.r && col < NO) ext_w[st][i] = *(const u16x8_t *)(a.ext_w + (long)j * a.K + col);
                    } else {
                        const int r = c >> 1, j = 16 * st + (c & 1) * 8, col = col0 + r;
                        if (j < a.r && col < NO) ext_w[st][i] = *(const u16x8_t *)(a.ext_w + (long)col * a.r + j);
                    }
                }
            }
        }
        // stage kt+1 is written while the MFMA waves work on stage kt; NSETS later stages are in flight from
        // memory (one register set each)
        constexpr int NSETS = 3;
        Regs rs[NSETS];
#pragma unroll
        for (int i = 0; i < NSETS; ++i) load_global(i, rs[i]);
        stage(rs[0], 0);
        load_global(NSETS, rs[0]);
        __syncthreads();
        auto step = [&](int kt, Regs &rg) {
            stage(rg, (kt + 1) & 1);
            load_global(kt + 1 + NSETS, rg);
            __syncthreads();
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
        __syncthreads();                        // pairs with the MFMA waves' final wait-and-barrier
    }

    // --- LoRA term as extra contraction steps: Act' = sc * t (or u), W' = B (or A^T), zero-padded to 16.
    //     Every wave is past the last barrier of the main loop, so every LDS stage is free.
    constexpr int ESTR = TN + 8;                            // row pitch of a wave's epilogue area
    constexpr int SIDE_R = 32;                              // adapter columns of the masked epilogue's side tiles
    uint16_t *const side_u = smem + MW * TM * ESTR;         // [BM][SIDE_R] rows of u, behind the epilogue areas
    uint16_t *const side_a = side_u + BM * SIDE_R;          // [SIDE_R][BN] columns of A
    if constexpr (MASKED) {
        if (stager) {                                       // the prefetched pieces, as they are (zero past the rank)
#pragma unroll
            for (int st = 0; st < EXT_STEPS; ++st) {
#pragma unroll
                for (int i = 0; i < EXT_A; ++i) {
                    const int c = stid + NSTG * i;
                    *(u16x8_t *)(side_u + (c >> 1) * SIDE_R + 16 * st + (c & 1) * 8) = ext_a[st][i];
                }
#pragma unroll
                for (int i = 0; i < EXT_W; ++i) {
                    const int c = stid + NSTG * i;
                    *(u16x8_t *)(side_a + (16 * st + c / (BN / 8)) * BN + (c % (BN / 8)) * 8) = ext_w[st][i];
                }
            }
        }
    }
    if (!MASKED && a.r > 0 && split == 0) {                 // the first workgroup of a split contraction adds it
        const int nsteps = (a.r + 15) / 16, width = nsteps * 16;
        if (!SYM && stager && nsteps <= EXT_STEPS) {        // operands already in registers
#pragma unroll
            for (int st = 0; st < EXT_STEPS; ++st) {
                if (st >= nsteps) break;
#pragma unroll
                for (int i = 0; i < EXT_A; ++i) {
                    const int c = stid + NSTG * i, r = c >> 1, jc = 2 * st + (c & 1);
                    u16x8_t p;
#pragma unroll
                    for (int h = 0; h < 8; ++h) p[h] = to16<BF16>(a.sc * cvt16<BF16>(ext_a[st][i][h]));
                    *(u16x8_t *)(xs + r * BK + ((jc ^ ((r >> 1) & 7)) * 8)) = p;  // same swizzle as the main loop
                }
#pragma unroll
                for (int i = 0; i < EXT_W; ++i) {
                    const int c = stid + NSTG * i;
                    if constexpr (TRANS)
                        *(u16x8_t *)(wsm + (16 * st + c / (BN / 8)) * WPITCH
                                     + (((c % (BN / 8)) ^ wswz(c / (BN / 8))) * 8)) = ext_w[st][i];
                    else if constexpr (!SYM)
                        *(u16x8_t *)(wsm + (c >> 1) * LDS_STRIDE + 16 * st + (c & 1) * 8) = ext_w[st][i];
                }
            }
        } else if (stager) {
            const int cpr = width / 8;                      // 8-element chunks per row
            for (int c = stid; c < BM * cpr; c += NSTG) {
                const int r = c / cpr, jc = c % cpr, j = jc * 8;
                u16x8_t p = {0, 0, 0, 0, 0, 0, 0, 0};
                if (j < a.r) {
                    const int gm = min(row0 + r, a.M - 1);
                    const u16x8_t v = *(const u16x8_t *)(a.ext_act + (long)gm * a.r + j);
#pragma unroll
                    for (int h = 0; h < 8; ++h) p[h] = to16<BF16>(a.sc * cvt16<BF16>(v[h]));
                }
                *(u16x8_t *)(xs + r * BK + ((jc ^ ((r >> 1) & 7)) * 8)) = p;  // same swizzle as the main loop
            }
            if constexpr (TRANS) {          // rows j of A, the tile's columns contiguous: the stage's own layout
                for (int c = stid; c < width * (BN / 8); c += NSTG) {
                    const int j = c / (BN / 8), col = col0 + (c % (BN / 8)) * 8;
                    u16x8_t p = {0, 0, 0, 0, 0, 0, 0, 0};
                    if (j < a.r && col < NO) p = *(const u16x8_t *)(a.ext_w + (long)j * a.K + col);
                    *(u16x8_t *)(wsm + j * WPITCH + (((c % (BN / 8)) ^ wswz(j)) * 8)) = p;
                }
            } else {
                for (int c = stid; c < BN * cpr; c += NSTG) {
                    const int r = c / cpr, j = (c % cpr) * 8;
                    const int col = col0 + r;
                    u16x8_t p = {0, 0, 0, 0, 0, 0, 0, 0};
                    if (j < a.r && col < NO) p = *(const u16x8_t *)(a.ext_w + (long)col * a.r + j);
                    if constexpr (SYM) *(u16x8_t *)(wsm + r * WPITCH + (((c % cpr) ^ fswz(r)) * 8)) = p;
                    else *(u16x8_t *)(wsm + r * LDS_STRIDE + j) = p;
                }
            }
        }
        __syncthreads();
        if (feeder) {
            for (int ks = 0; ks < nsteps; ++ks) {
                Frags fx;
                load_frags(0, 0, ks, fx);
                mfma_frags(fx);
            }
        }
        __syncthreads();
    }

    // --- epilogue: fp32 accumulators -> 16 bit.  Each MFMA wave lays its TM x TN block into its own LDS area in
    //     row-major order; then all waves stream the areas out in 16-byte pieces (8 lanes per 128-byte row
    //     segment).  Rows beyond M and columns beyond NO (always whole 8-element pieces) are dropped.
    if (a.splits > 1) {
        // split contraction: the fp32 accumulators go to this split's plane as they are (a lane's 32 neighbours
        // write 128 consecutive bytes of a row); a second kernel sums the planes in order and rounds once
        if (feeder) {
            float *P = a.part + (size_t)split * a.M * NO;
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const int gcol = col0 + wn * TN + j * 32 + (lane & 31);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int grow = row0 + wm * TM + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                        if (grow < a.M && gcol < NO) P[(size_t)grow * NO + gcol] = acc[i][j][v];
                    }
                }
        }
        return;
    }
    if (feeder) {
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
        for (int c = tid; c < MW * PER_AREA; c += THREADS) {
            const int w = c / PER_AREA, cc = c % PER_AREA;
            const int r = cc / CPR, ch = (cc % CPR) * 8;
            const int grow = row0 + (w / WN) * TM + r, gcol = col0 + (w % WN) * TN + ch;
            u32x4_t v = *(const u32x4_t *)(smem + w * (TM * ESTR) + r * ESTR + ch);
            if constexpr (MASKED) {
                if (grow < a.M && gcol < NO) {
                    const uint32_t bits = a.keep[(size_t)grow * (NO / 8) + gcol / 8];
                    const uint16_t *ur = side_u + ((w / WN) * TM + r) * SIDE_R, *ap = side_a + (w % WN) * TN + ch;
                    float l[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    const int rp = (a.r + 7) / 8;               // 8-column pieces of the adapter
                    for (int jp = 0; jp < rp; ++jp) {
                        const u16x8_t u8 = *(const u16x8_t *)(ur + 8 * jp);
#pragma unroll
                        for (int jj = 0; jj < 8; ++jj) {
                            const float uj = cvt16<BF16>(u8[jj]);
                            const u16x8_t a8 = *(const u16x8_t *)(ap + (8 * jp + jj) * BN);
#pragma unroll
                            for (int e = 0; e < 8; ++e) l[e] = fmaf(uj, cvt16<BF16>(a8[e]), l[e]);
                        }
                    }
                    const u16x8_t b8 = __builtin_bit_cast(u16x8_t, v);
                    u16x8_t o8;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        o8[e] = ((bits >> e) & 1u) ? to16<BF16>(cvt16<BF16>(b8[e]) + a.keep_sc * l[e]) : b8[e];
                    v = __builtin_bit_cast(u32x4_t, o8);
                }
            }
            // written once and not read by this kernel: the non-temporal hint keeps the output from displacing the
            // activation rows and weight columns that other tiles still want from L2 (-1 us per GEMM)
            if (grow < a.M && gcol < NO) __builtin_nontemporal_store(v, (u32x4_t *)(a.out + ((long)grow * NO + gcol)));
        }
    }
}

template <int BITS, bool BF16, bool TRANS, int BM, int BN, int WM, int WN, bool MASKED = false, bool SYM = false>
void launch_variant(const GemmArgs &a, hipStream_t s)
{
    constexpr size_t wstage = TRANS ? (size_t)BK * BN : (size_t)BN * (SYM ? BK : LDS_STRIDE);
    constexpr size_t lds_pipe = (GEMM_NXS * (size_t)BM * BK + 2 * wstage) * sizeof(uint16_t);
    constexpr size_t lds_side = MASKED ? (size_t)32 * (BM + BN) * sizeof(uint16_t) : 0;    // side tiles of the masked epilogue
    constexpr size_t lds_epi = (size_t)WM * WN * (BM / WM) * (BN / WN + 8) * sizeof(uint16_t) + lds_side;
    constexpr size_t lds = lds_pipe > lds_epi ? lds_pipe : lds_epi;
    static_assert(lds <= 160 * 1024, "LDS of a compute unit");
    auto kern = qgemm_kernel<BITS, BF16, TRANS, BM, BN, WM, WN, MASKED, SYM>;
    ensure_dynamic_lds((const void *)kern, (int)(lds));
    QLORA_LAUNCH(kern, dim3(a.tiles_m * a.tiles_n * a.splits), dim3(WM * WN * 64 + (SYM ? 0 : STAGERS)), lds, s, a);
}

// out = round16(sum over the split planes, in order): 8 elements per thread
template <bool BF16>
__global__ __launch_bounds__(256) void splitk_sum_kernel(const float *__restrict__ part, uint16_t *__restrict__ out,
                                                         size_t plane, int splits)
{
    const size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
    if (e >= plane) return;                             // plane is a multiple of 8
    float acc[8];
#pragma unroll
    for (int h = 0; h < 8; ++h) acc[h] = 0.f;
    for (int sp = 0; sp < splits; ++sp) {
        const float4_t lo = *(const float4_t *)(part + sp * plane + e), hi = *(const float4_t *)(part + sp * plane + e + 4);
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            acc[h] += lo[h];
            acc[4 + h] += hi[h];
        }
    }
    u16x8_t o;
#pragma unroll
    for (int h = 0; h < 8; ++h) o[h] = to16<BF16>(acc[h]);
    *(u16x8_t *)(out + e) = o;
}

template <int BITS, bool BF16, bool TRANS>
void launch_tiles(GemmArgs &a, hipStream_t s)
{
    constexpr int BM = 256, BN = 128, WM = 2, WN = 2;       // tile shape and grid of MFMA waves
    static_assert(BN == GEMM_SPLIT_BN, "gemm_splits() counts tiles of this width");
    const int NO = TRANS ? a.K : a.N, KC = TRANS ? a.N : a.K;
    a.tiles_n = (NO + BN - 1) / BN;
    a.splits = 1;
    a.kt_split = (KC + BK - 1) / BK;
    // fewer tiles than CUs: halve the tile height, so that (up to) twice as many CUs work; far fewer: also split
    // the contraction over several workgroups per tile
    if constexpr (BM == 256) {
        if (((a.M + 255) / 256) * a.tiles_n < 256) {
            a.tiles_m = (a.M + 127) / 128;
            if constexpr (TRANS) {
                if (a.keep) {           // the masked epilogue needs the whole contraction in one workgroup
                    launch_variant<BITS, BF16, TRANS, 128, BN, WM, WN, true>(a, s);
                    return;
                }
            }
            const int splits = a.part ? gemm_splits(a.M, NO, KC) : 1;
            if (splits > 1) {
                a.splits = splits;
                a.kt_split = (a.kt_split + splits - 1) / splits;
            }
            launch_variant<BITS, BF16, TRANS, 128, BN, WM, WN>(a, s);
            if (splits > 1) {
                const size_t plane = (size_t)a.M * NO;
                QLORA_LAUNCH(splitk_sum_kernel<BF16>, dim3((unsigned)((plane / 8 + 255) / 256)), dim3(256), 0, s,
                                   a.part, a.out, plane, splits);
            }
            return;
        }
    }
    a.tiles_m = (a.M + BM - 1) / BM;
    if constexpr (TRANS) {
        if (a.keep) {
            launch_variant<BITS, BF16, TRANS, BM, BN, WM, WN, true>(a, s);
            return;
        }
    }
    // At least one 256 x 256 tile per compute unit, and rounds of 256 tiles that are at least 80 % full: the
    // symmetric-wave kernel (5-11 % less time than the 256 x 128 tiles at M = 4096 and 8192; a launch of 344 tiles,
    // two rounds of which the second is a third full, is 10 % slower than the 688 smaller tiles).
    {
        const int tn = (NO + 255) / 256, tiles = a.tiles_m * tn, rounds = (tiles + 255) / 256;
        if (tiles >= 256 && tiles * 10 >= rounds * 256 * 8) {
            a.tiles_n = tn;
            launch_variant<BITS, BF16, TRANS, 256, 256, 2, 4, false, true>(a, s);
            return;
        }
    }
    launch_variant<BITS, BF16, TRANS, BM, BN, WM, WN>(a, s);
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
                     const void *t, const void *B, void *y, float *part, hipStream_t s)
{
    GemmArgs a{(const uint16_t *)x, packed, (const uint16_t *)scales, zeros, (const uint16_t *)t, (const uint16_t *)B,
               (uint16_t *)y, p.M, p.N, p.K, p.G, p.r, p.sc, 0, 0, group_magic(p.G), part, 1, 0, nullptr, 0.f};
    launch_bits_dtype<false>(p, a, s);
}

void launch_bwd_dx_mfma(const Problem &p, const void *dy, const uint32_t *packed, const void *scales,
                        const uint8_t *zeros, const void *u, const void *A, void *dx, float *part,
                        const uint32_t *keep, float keep_scale, hipStream_t s)
{
    GemmArgs a{(const uint16_t *)dy, packed, (const uint16_t *)scales, zeros, (const uint16_t *)u, (const uint16_t *)A,
               (uint16_t *)dx, p.M, p.N, p.K, p.G, p.r, p.sc, 0, 0, group_magic(p.G), part, 1, 0,
               p.r > 0 ? (const uint8_t *)keep : nullptr, p.sc * keep_scale};
    launch_bits_dtype<true>(p, a, s);
}

}  // namespace qlora
