// The LREC objective and its gradient with respect to the student logits (Sec. 3.2 "Optimization", Eq. 1 and 2):
//
//   per token   y_hat = softmax(student logits),  y = softmax(teacher logits)
//               KL = sum_i y_hat_i (log y_hat_i - log y_i)          (student first, as the paper writes it)
//               CE = -log y_hat[label]                               (next-token cross entropy; none if label < 0)
//   objective   mean over the M tokens of lambda_KL KL + lambda_CE CE
//   gradient    d objective / d z_k = (lambda_KL y_hat_k (d_k - KL) + lambda_CE (y_hat_k - [k = label])) / M,
//               d_k = log y_hat_k - log y_k
//
// The work is a reduction over a 32000-wide vocabulary per token: three sweeps over the row (log-sum-exp of both
// rows, KL, gradient).  It is bound by HBM: both rows are read once (a workgroup keeps its token's two rows in
// registers, 16-bit, for all three sweeps) and the gradient is written once, 6 bytes per logit in all.
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
};

// (max, sum of exp(v - max)) pairs are merged; the neutral element is (-inf, 0)
struct MaxSum {
    float m, s;
};
__device__ __forceinline__ MaxSum merge(MaxSum a, MaxSum b)
{
    const float m = fmaxf(a.m, b.m);
    if (m == -INFINITY) return MaxSum{m, 0.f};
    return MaxSum{m, a.s * fast_exp2((a.m - m) * LOG2E) + b.s * fast_exp2((b.m - m) * LOG2E)};
}
__device__ __forceinline__ MaxSum wave_merge(MaxSum v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        MaxSum o{__shfl_xor(v.m, off, WAVE), __shfl_xor(v.s, off, WAVE)};
        v = merge(v, o);
    }
    return v;
}

// CH > 0: the thread's CH 8-element pieces of both rows stay in registers; CH == 0: every sweep reads them again
template <bool BF16, int CH>
__global__ __launch_bounds__(LT) void lrec_loss_kernel(const LossArgs a)
{
    __shared__ MaxSum red_ms[2][LT / 64];
    __shared__ float red_f[LT / 64];
    __shared__ float bc[4];              // lse of the student row, lse of the teacher row, KL
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
            rs[i] = *(const u16x8_t *)(zs + 8 * (long)p);
            rt[i] = *(const u16x8_t *)(zt + 8 * (long)p);
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

    // sweep 1: log-sum-exp of both rows.  The thread's own maxima first (fp16: packed, exact), so that every logit
    // costs one exponential and the (max, sum) pairs are merged once per thread, not once per piece.
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
            const u32x4_t sw = __builtin_bit_cast(u32x4_t, s8), tw = __builtin_bit_cast(u32x4_t, t8);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                hs = __builtin_elementwise_max(hs, __builtin_bit_cast(half2_t, sw[e]));
                ht = __builtin_elementwise_max(ht, __builtin_bit_cast(half2_t, tw[e]));
            }
        }
        ls = fmaxf((float)hs[0], (float)hs[1]);
        lt = fmaxf((float)ht[0], (float)ht[1]);
    }
    float ss = 0.f, st = 0.f;
    {
        const float os = -ls * LOG2E, ot = -lt * LOG2E;       // exp(v - max) = exp2(v log2e - max log2e)
#pragma unroll CH > 0 ? CH : 1
        for (int i = 0; i < my_pieces; ++i) {
            if (piece_of(i) >= pieces) break;
            u16x8_t s8, t8;
            get(i, s8, t8);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                ss += fast_exp2(fmaf(val(s8, e), LOG2E, os));
                st += fast_exp2(fmaf(val(t8, e), LOG2E, ot));
            }
        }
    }
    MaxSum ms = wave_merge(MaxSum{ls, ss}), mt = wave_merge(MaxSum{lt, st});
    if (lane == 0) {
        red_ms[0][wave] = ms;
        red_ms[1][wave] = mt;
    }
    __syncthreads();
    if (tid < 2) {
        MaxSum v = red_ms[tid][0];
#pragma unroll
        for (int w = 1; w < LT / 64; ++w) v = merge(v, red_ms[tid][w]);
        bc[tid] = v.m + __builtin_amdgcn_logf(v.s) * LN2;     // the hardware's log2
    }
    __syncthreads();
    const float lse_s = bc[0], lse_t = bc[1];
    const float delta = lse_s - lse_t;                        // d_i = log y_hat_i - log y_i = (zs_i - zt_i) - delta
    const float off_s = -lse_s * LOG2E;                       // y_hat_i = exp2(zs_i log2e + off_s)

    // sweep 2: KL = sum_i y_hat_i d_i = sum_i y_hat_i (zs_i - zt_i) - delta sum_i y_hat_i; the last sum is carried
    // along (it is 1 up to rounding).  y_hat and zs - zt are kept, as fp16 pairs (2^-11 relative), for the gradient
    // sweep: they take the registers of the piece they were computed from.  `one` is 1.0 the compiler cannot see through: zs * one - zt then stays one mixed-precision fma on the
    // two halves instead of two conversions and a subtraction.
    float one = 1.f, zero = 0.f;
    asm volatile("" : "+v"(one), "+v"(zero));
    float kl = 0.f, psum = 0.f;
#pragma unroll CH > 0 ? CH : 1
    for (int i = 0; i < my_pieces; ++i) {
        if (piece_of(i) >= pieces) break;
        u16x8_t s8, t8;
        get(i, s8, t8);
        half8_t ph, dh;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float pe = fast_exp2(fmaf(val(s8, e), LOG2E, off_s));
            const float de = fmaf(val(s8, e), one, -val(t8, e));
            kl = fmaf(pe, de, kl);
            psum += pe;
            ph[e] = (half_t)pe;
            dh[e] = (half_t)de;
        }
        if constexpr (CH > 0) {
            rs[i] = __builtin_bit_cast(u16x8_t, ph);
            rt[i] = __builtin_bit_cast(u16x8_t, dh);
        }
    }
    kl = wave_sum(fmaf(-delta, psum, kl));
    if (lane == 0) red_f[wave] = kl;
    __syncthreads();
    const int label = a.labels[row];
    const bool has = label >= 0 && label < a.V;
    if (tid == 0) {
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < LT / 64; ++w) v += red_f[w];
        bc[2] = v;
        const float ce = has ? lse_s - cvt16<BF16>(zs[label]) : 0.f;
        if (a.kl) a.kl[row] = v;
        if (a.ce) a.ce[row] = ce;
        a.tok[row] = a.lkl * v + a.lce * ce;
    }
    if (!a.grad) return;
    __syncthreads();
    // sweep 3: the gradient row, g_i = y_hat_i (c1 (zs_i - zt_i) + c2) - [i = label] lce / M
    const float inv_m = 1.f / (float)a.M, lce = has ? a.lce : 0.f;
    const float c1 = a.lkl * inv_m, c2 = (lce - a.lkl * (bc[2] + delta)) * inv_m;
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
                            fmaf((float)__builtin_bit_cast(half8_t, rt[i])[e], c1, c2), zero);
            else
                g[e] = fast_exp2(fmaf(val(s8, e), LOG2E, off_s)) * fmaf(fmaf(val(s8, e), one, -val(t8, e)), c1, c2);
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) g8[e] = to16<BF16>(g[e]);
        *(u16x8_t *)(grow + k0) = g8;
    }
    // the target's own entry carries one more term, -lce / M: the thread that wrote it (same thread, so the two
    // stores to that address stay in order) computes it again in full and overwrites it
    if (has && ((label >> 3) % LT) == tid) {
        const float z = cvt16<BF16>(zs[label]), t = cvt16<BF16>(zt[label]);
        float p, d;
        if constexpr (CH > 0) {       // the values the sweep used: y_hat and zs - zt as the fp16 they were kept in
            p = (float)(half_t)fast_exp2(fmaf(z, LOG2E, off_s));
            d = (float)(half_t)(z - t);
        } else {
            p = fast_exp2(fmaf(z, LOG2E, off_s));
            d = z - t;
        }
        grow[label] = to16<BF16>(fmaf(p, fmaf(d, c1, c2), zero) - lce * inv_m);
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
    if (per_thread <= 1) hipLaunchKernelGGL((lrec_loss_kernel<BF16, 1>), grid, block, 0, s, a);
    else if (per_thread <= 2) hipLaunchKernelGGL((lrec_loss_kernel<BF16, 2>), grid, block, 0, s, a);
    else if (per_thread <= 4) hipLaunchKernelGGL((lrec_loss_kernel<BF16, 4>), grid, block, 0, s, a);
    else if (per_thread <= 8) hipLaunchKernelGGL((lrec_loss_kernel<BF16, 8>), grid, block, 0, s, a);
    else if (per_thread <= 16) hipLaunchKernelGGL((lrec_loss_kernel<BF16, 16>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((lrec_loss_kernel<BF16, 0>), grid, block, 0, s, a);
}

}  // namespace

void launch_lrec_loss(const void *student, const void *teacher, const int32_t *labels, float lambda_kl,
                      float lambda_ce, float *kl, float *ce, float *tok, float *loss_mean, void *grad, int M, int V,
                      bool bf16, hipStream_t s)
{
    const LossArgs a{(const uint16_t *)student, (const uint16_t *)teacher, labels, kl, ce, tok, (uint16_t *)grad, M, V,
                     lambda_kl, lambda_ce};
    if (bf16)
        launch_loss<true>(a, s);
    else
        launch_loss<false>(a, s);
    hipLaunchKernelGGL(lrec_mean_kernel, dim3(1), dim3(256), 0, s, tok, loss_mean, M);
}

}  // namespace qlora
