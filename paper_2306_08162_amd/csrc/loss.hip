// The LREC objective and its gradient with respect to the student logits (Sec. 3.2 "Optimization", Eq. 1 and 2):
//
//   per token   y_hat = softmax(student logits),  y = softmax(teacher logits)
//               KL = sum_i y_hat_i (log y_hat_i - log y_i)          (student first, as the paper writes it)
//               CE = -log y_hat[label]                               (next-token cross entropy; none if label < 0)
//   objective   mean over the M tokens of lambda_KL KL + lambda_CE CE
//   gradient    d objective / d z_k = (lambda_KL y_hat_k (d_k - KL) + lambda_CE (y_hat_k - [k = label])) / M,
//               d_k = log y_hat_k - log y_k
//
// The work is a reduction over a 32000-wide vocabulary per token and is bound by HBM: both rows are read once and
// the gradient is written once, 6 bytes per logit in all.  Two sweeps over registers do it.  With e_i =
// exp(zs_i - m), m any upper bound of the row, and S = sum e_i:  y_hat_i = e_i / S  and
//     KL = sum_i y_hat_i ((zs_i - zt_i) - delta) = Q / S - delta,   Q = sum_i e_i (zs_i - zt_i),
//     delta = lse(zs) - lse(zt),
// so one sweep with one exponential per logit yields (m, S, Q) of the student row and (m, S) of the teacher row,
// merged over the threads like any running softmax; the second sweep forms the gradient from e_i and zs_i - zt_i,
// which the first one left behind in the registers the logits came in (as fp16).
#include "common.hpp"
#include "kernels.hpp"

namespace qlora {

namespace {

constexpr int LT = 512;              // threads per workgroup, one token row each
constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

// 2^x by the hardware instruction alone: results below 2^-126 come out as zero, which is what a softmax term that
// small is worth; the library routine's handling of that range costs five more instructions per call
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

struct LossArgs {
    const uint16_t *zs, *zt;         // student / teacher logits [M,V]
    const int32_t *labels;           // [M]
    float *kl, *ce;                  // [M] each, may be NULL
    float *tok;                      // [M] lambda_KL KL + lambda_CE CE
    uint16_t *grad;                  // [M,V], may be NULL
    int M, V;
    float lkl, lce;
    float gscale;                    // loss scaling: the gradient is written multiplied by this factor
};

// Running softmax state: m an upper bound of the values seen, s = sum exp(v - m), q = sum exp(v - m) w for a weight
// w per value (the student row carries w = zs - zt; the teacher row carries none).  The neutral element is (-inf, 0, 0).
struct SoftState {
    float m, s, q;
};
__device__ __forceinline__ SoftState merge(SoftState a, SoftState b)
{
    const float m = fmaxf(a.m, b.m);
    if (m == -INFINITY) return SoftState{m, 0.f, 0.f};
    const float fa = fast_exp2((a.m - m) * LOG2E), fb = fast_exp2((b.m - m) * LOG2E);
    return SoftState{m, a.s * fa + b.s * fb, a.q * fa + b.q * fb};
}
__device__ __forceinline__ SoftState wave_merge(SoftState v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        SoftState o{__shfl_xor(v.m, off, WAVE), __shfl_xor(v.s, off, WAVE), __shfl_xor(v.q, off, WAVE)};
        v = merge(v, o);
    }
    return v;
}

// CH > 0: the thread's CH 8-element pieces of both rows stay in registers; CH == 0: every sweep reads them again
template <bool BF16, int CH>
__global__ __launch_bounds__(LT) void lrec_loss_kernel(const LossArgs a)
{
    __shared__ SoftState red[2][LT / 64];
    __shared__ float bc[4];              // max and sum of the student row, delta, KL
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int pieces = a.V / 8;
    const uint16_t *zs = a.zs + (long)row * a.V, *zt = a.zt + (long)row * a.V;
    constexpr int NCH = CH > 0 ? CH : 1;
    u16x8_t rs[NCH], rt[NCH];
    const int my_pieces = CH > 0 ? CH : (pieces + LT - 1) / LT;
    auto piece_of = [&](int i) { return tid + LT * i; };
    auto get = [&](int i, u16x8_t &s8, u16x8_t &t8) {
        if constexpr (CH > 0) {
            s8 = rs[i];
            t8 = rt[i];
        } else {
            s8 = *(const u16x8_t *)(zs + 8 * (long)piece_of(i));
            t8 = *(const u16x8_t *)(zt + 8 * (long)piece_of(i));
        }
    };
    if constexpr (CH > 0) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int p = piece_of(i) < pieces ? piece_of(i) : 0;          // the row's first piece stands in past the end
            // read once, never again: the non-temporal hint keeps the 393 MB of a call from displacing each other
            // in the caches on their way through (83 -> 76 us at 2048 x 32000)
            rs[i] = __builtin_nontemporal_load((const u16x8_t *)(zs + 8 * (long)p));
            rt[i] = __builtin_nontemporal_load((const u16x8_t *)(zt + 8 * (long)p));
        }
    }

    // A logit as fp32.  For fp16 the conversion is written as a cast of the half, so that it folds into the
    // mixed-precision fma that consumes it; bf16 is a shift.
    auto val = [](const u16x8_t &v, int e) -> float {
        if constexpr (BF16)
            return bf16_bits_to_f32(v[e]);
        else
            return (float)__builtin_bit_cast(half8_t, v)[e];
    };

    // sweep 1.  The thread's own maxima first (fp16: packed, exact), then one exponential per logit.  `one` is 1.0
    // the compiler cannot see through: zs * one - zt then stays one mixed-precision fma on the two halves instead of
    // two conversions and a subtraction.
    float one = 1.f, zero = 0.f;
    asm volatile("" : "+v"(one), "+v"(zero));
    float ls = -INFINITY, lt = -INFINITY;
    if constexpr (BF16) {
#pragma unroll CH > 0 ? CH : 1
        for (int i = 0; i < my_pieces; ++i) {
            if (piece_of(i) >= pieces) break;
            u16x8_t s8, t8;
            get(i, s8, t8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                ls = fmaxf(ls, val(s8, e));
                lt = fmaxf(lt, val(t8, e));
            }
        }
    } else {
        const half_t lowest = (half_t)-65504.f;
        half2_t hs = {lowest, lowest}, ht = {lowest, lowest};
#pragma unroll CH > 0 ? CH : 1
        for (int i = 0; i < my_pieces; ++i) {
            if (piece_of(i) >= pieces) break;
            u16x8_t s8, t8;
            get(i, s8, t8);
            // (written out pair by pair: a loop over the four 32-bit words, bit-cast one at a time, was compiled
            // down to its first iteration by this toolchain)
            const half8_t sh = __builtin_bit_cast(half8_t, s8), th = __builtin_bit_cast(half8_t, t8);
            const half2_t s01 = {sh[0], sh[1]}, s23 = {sh[2], sh[3]}, s45 = {sh[4], sh[5]}, s67 = {sh[6], sh[7]};
            const half2_t t01 = {th[0], th[1]}, t23 = {th[2], th[3]}, t45 = {th[4], th[5]}, t67 = {th[6], th[7]};
            hs = __builtin_elementwise_max(hs, __builtin_elementwise_max(__builtin_elementwise_max(s01, s23),
                                                                         __builtin_elementwise_max(s45, s67)));
            ht = __builtin_elementwise_max(ht, __builtin_elementwise_max(__builtin_elementwise_max(t01, t23),
                                                                         __builtin_elementwise_max(t45, t67)));
        }
        ls = fmaxf((float)hs[0], (float)hs[1]);
        lt = fmaxf((float)ht[0], (float)ht[1]);
    }
    float ss = 0.f, st = 0.f, qs = 0.f;
    const float os = -ls * LOG2E, ot = -lt * LOG2E;           // exp(v - max) = exp2(v log2e - max log2e)
#pragma unroll CH > 0 ? CH : 1
    for (int i = 0; i < my_pieces; ++i) {
        if (piece_of(i) >= pieces) break;
        u16x8_t s8, t8;
        get(i, s8, t8);
        half8_t eh, dh;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float es = fast_exp2(fmaf(val(s8, e), LOG2E, os));
            const float dz = fmaf(val(s8, e), one, -val(t8, e));
            ss += es;
            qs = fmaf(es, dz, qs);
            st += fast_exp2(fmaf(val(t8, e), LOG2E, ot));
            eh[e] = (half_t)es;
            // kept as fp16: a masked student logit (-65504) against an ordinary teacher logit would round to -inf
            // and turn its zero gradient entry, 0 * inf, into a NaN
            dh[e] = (half_t)__builtin_amdgcn_fmed3f(dz, -65504.f, 65504.f);
        }
        if constexpr (CH > 0) {       // e_i and zs_i - zt_i (2^-11 relative) take the place of the logits
            rs[i] = __builtin_bit_cast(u16x8_t, eh);
            rt[i] = __builtin_bit_cast(u16x8_t, dh);
        }
    }
    const SoftState ws = wave_merge(SoftState{ls, ss, qs}), wt = wave_merge(SoftState{lt, st, 0.f});
    if (lane == 0) {
        red[0][wave] = ws;
        red[1][wave] = wt;
    }
    __syncthreads();
    const int label = a.labels[row];
    const bool has = label >= 0 && label < a.V;
    if (tid == 0) {
        SoftState vs = red[0][0], vt = red[1][0];
#pragma unroll
        for (int w = 1; w < LT / 64; ++w) {
            vs = merge(vs, red[0][w]);
            vt = merge(vt, red[1][w]);
        }
        const float lse_s = vs.m + __builtin_amdgcn_logf(vs.s) * LN2;      // the hardware's log2
        const float lse_t = vt.m + __builtin_amdgcn_logf(vt.s) * LN2;
        const float delta = lse_s - lse_t;
        const float klv = vs.q / vs.s - delta;
        const float ce = has ? lse_s - cvt16<BF16>(zs[label]) : 0.f;
        bc[0] = vs.m;
        bc[1] = vs.s;
        bc[2] = delta;
        bc[3] = klv;
        if (a.kl) a.kl[row] = klv;
        if (a.ce) a.ce[row] = ce;
        a.tok[row] = a.lkl * klv + a.lce * ce;
    }
    if (!a.grad) return;
    __syncthreads();
    // sweep 2: the gradient row, g_i = y_hat_i (c1 (zs_i - zt_i) + c2) - [i = label] lce / M, with
    // y_hat_i = e_i phi, phi = exp(ls - m) / S the thread's share of the normalisation
    const float row_m = bc[0], row_s = bc[1], delta = bc[2], klv = bc[3];
    const float inv_m = a.gscale / (float)a.M, lce = has ? a.lce : 0.f;   // 1/M of the mean, times the loss scale
    const float c1 = a.lkl * inv_m, c2 = (lce - a.lkl * (klv + delta)) * inv_m;
    const float phi = fast_exp2((ls - row_m) * LOG2E) / row_s;
    const float c1p = c1 * phi, c2p = c2 * phi;
    const float off_s = -(row_m + __builtin_amdgcn_logf(row_s) * LN2) * LOG2E;   // y_hat_i = exp2(zs_i log2e + off_s)
    uint16_t *grow = a.grad + (long)row * a.V;
#pragma unroll CH > 0 ? CH : 1
    for (int i = 0; i < my_pieces; ++i) {
        if (piece_of(i) >= pieces) break;
        u16x8_t s8, t8, g8;
        if constexpr (CH == 0) get(i, s8, t8);
        const int k0 = 8 * piece_of(i);
        float g[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            if constexpr (CH > 0)
                g[e] = fmaf((float)__builtin_bit_cast(half8_t, rs[i])[e],
                            fmaf((float)__builtin_bit_cast(half8_t, rt[i])[e], c1p, c2p), zero);
            else
                g[e] = fast_exp2(fmaf(val(s8, e), LOG2E, off_s)) * fmaf(fmaf(val(s8, e), one, -val(t8, e)), c1, c2);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) g8[e] = to16<BF16>(g[e]);
        __builtin_nontemporal_store(g8, (u16x8_t *)(grow + k0));
    }
    // the target's own entry carries one more term, -lce / M: the thread that wrote it (same thread, so the two
    // stores to that address stay in order) computes it again in full and overwrites it
    if (has && ((label >> 3) % LT) == tid) {
        const float z = cvt16<BF16>(zs[label]), t = cvt16<BF16>(zt[label]);
        float gl;
        if constexpr (CH > 0)         // from the values the sweep used: e and zs - zt as the fp16 they were kept in
            gl = fmaf((float)(half_t)fast_exp2(fmaf(z, LOG2E, os)),
                      fmaf((float)(half_t)__builtin_amdgcn_fmed3f(z - t, -65504.f, 65504.f), c1p, c2p), zero);
        else
            gl = fast_exp2(fmaf(z, LOG2E, off_s)) * fmaf(z - t, c1, c2);
        grow[label] = to16<BF16>(gl - lce * inv_m);
    }
}

// mean of the per-token values, summed in a fixed order by one workgroup
__global__ __launch_bounds__(256) void lrec_mean_kernel(const float *__restrict__ tok, float *__restrict__ out, int M)
{
    __shared__ float red[256];
    float v = 0.f;
    for (int i = threadIdx.x; i < M; i += 256) v += tok[i];
    red[threadIdx.x] = v;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = red[0] / (float)M;
}

template <bool BF16>
void launch_loss(const LossArgs &a, hipStream_t s)
{
    const int per_thread = (a.V / 8 + LT - 1) / LT;
    const dim3 grid(a.M), block(LT);
    if (per_thread <= 1) QLORA_LAUNCH((lrec_loss_kernel<BF16, 1>), grid, block, 0, s, a);
    else if (per_thread <= 2) QLORA_LAUNCH((lrec_loss_kernel<BF16, 2>), grid, block, 0, s, a);
    else if (per_thread <= 4) QLORA_LAUNCH((lrec_loss_kernel<BF16, 4>), grid, block, 0, s, a);
    else if (per_thread <= 8) QLORA_LAUNCH((lrec_loss_kernel<BF16, 8>), grid, block, 0, s, a);
    else if (per_thread <= 16) QLORA_LAUNCH((lrec_loss_kernel<BF16, 16>), grid, block, 0, s, a);
    else QLORA_LAUNCH((lrec_loss_kernel<BF16, 0>), grid, block, 0, s, a);
}

}  // namespace

void launch_lrec_loss(const void *student, const void *teacher, const int32_t *labels, float lambda_kl,
                      float lambda_ce, float grad_scale, float *kl, float *ce, float *tok, float *loss_mean, void *grad,
                      int M, int V, bool bf16, hipStream_t s)
{
    const LossArgs a{(const uint16_t *)student, (const uint16_t *)teacher, labels, kl, ce, tok, (uint16_t *)grad, M, V,
                     lambda_kl, lambda_ce, grad_scale};
    if (bf16)
        launch_loss<true>(a, s);
    else
        launch_loss<false>(a, s);
    QLORA_LAUNCH(lrec_mean_kernel, dim3(1), dim3(256), 0, s, tok, loss_mean, M);
}

}  // namespace qlora
