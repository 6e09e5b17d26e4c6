// Host-side launchers of the HIP kernels; one translation unit per kernel family.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace qlora {

// One quantized LoRA linear problem, already validated by the C ABI layer.
struct Problem {
    int M, N, K;
    int bits, G, r;
    float sc;     // alpha / r (0 when r == 0)
    bool bf16;    // activation / adapter dtype
};

// Kernels that use more than 64 KB of dynamic LDS must have that ceiling raised once per function and device; safe to
// call from several host threads.
void ensure_dynamic_lds(const void *kernel, int bytes);

// Launch bookkeeping of the calling host thread: every kernel launch of the library goes through QLORA_LAUNCH, which
// asks the runtime for the launch's status right away and keeps the first failure.  An entry point clears both the
// runtime's sticky error and this record before its first launch (an error left behind by somebody else's earlier
// call is not this call's) and reports the record when it returns.
void launch_errors_clear();
void launch_errors_note();          // after a launch (or a runtime call that may fail): keep the first error
bool launch_errors_seen();
#define QLORA_LAUNCH(...)                \
    do {                                 \
        hipLaunchKernelGGL(__VA_ARGS__); \
        ::qlora::launch_errors_note();   \
    } while (0)

// pack.hip
void launch_pack(const uint8_t *codes, uint32_t *packed, int N, int K, int bits, hipStream_t s);
void launch_unpack(const uint32_t *packed, uint8_t *codes, int N, int K, int bits, hipStream_t s);
// zero-points [N, groups] <-> their bit-packed form [N, ceil(groups*bits/32)] (same stream convention as the codes)
void launch_pack_zeros(const uint8_t *zeros, uint32_t *packed, int N, int groups, int bits, hipStream_t s);
void launch_unpack_zeros(const uint32_t *packed, uint8_t *zeros, int N, int groups, int bits, hipStream_t s);
// column j of the packed matrix takes the codes of column perm[j] (zero codes where perm[j] is outside [0, K))
void launch_pack_permuted(const uint8_t *codes, const int32_t *perm, uint32_t *packed, int N, int K, int bits,
                          hipStream_t s);
// dst[m, j] = src[m, index[j]], 16-bit elements, K % 8 == 0 (0 where index[j] is outside [0, K))
void launch_gather_columns(const void *src, const int32_t *index, void *dst, int M, int K, hipStream_t s);
// benchmark instrumentation: 1024 partial exclusive-ors of the 32-bit words of a buffer, read once with 16-byte loads
void launch_stream_probe(const void *src, size_t bytes, uint32_t *out, hipStream_t s);
// benchmark instrumentation: iters x 8 register-resident 32x32x16 fp16 MFMAs per wave, 256 workgroups of 8 waves
void launch_mfma_probe(float *out, int iters, bool random, hipStream_t s);

// adapters.hip -- the rank-r side products and the adapter gradients
// t[M,r] = x[M,K] A[r,K]^T; with a keep mask (LoRA dropout, one bit per element of x, bit k % 32 of word k / 32 of
// the row) t = keep_scale * (x * keep) A^T
// planes != NULL, no mask and at most LORA_DOWN_SMALL_MAX_M token rows: the contraction is split over workgroups
// (planes holds lora_down_small_planes(K) * M * r floats), two launches.
constexpr int LORA_DOWN_SMALL_MAX_M = 32;
int lora_down_small_planes(int K);
void launch_lora_down(const void *x, const void *A, void *t, int M, int K, int r, bool bf16, const uint32_t *keep,
                      float keep_scale, hipStream_t s, float *planes = nullptr);
// dx[m,k] += f * keep[m,k] * sum_j u[m,j] A[j,k]: the adapter's share of dX under dropout, on top of the base product
void launch_lora_dx_masked(void *dx, const void *u, const void *A, const uint32_t *keep, int M, int K, int r, float f,
                           bool bf16, hipStream_t s);
// u[M,r] = dy[M,N] B[N,r]
void launch_lora_u(const void *dy, const void *B, void *u, int M, int N, int r, bool bf16, hipStream_t s);
// dB[N,r] = sc * dy[M,N]^T t[M,r] and dA[r,K] = sc * u[M,r]^T x[M,K], one launch for both, sums in a fixed order.
// beta != 0: dB = beta*dB + ..., dA likewise.  keep != NULL (LoRA dropout): x stands for keep_scale * x * keep in dA.
// Stacked adapters: t and u are [M, r_all], the first `frozen` adapter columns have no gradient, r = r_all - frozen,
// dB is [N, r], dA [r, K].
void launch_adapter_grads(const void *dy, const void *t, const void *x, const void *u, float *dB, float *dA, int M, int N,
                          int K, int r_all, int frozen, float sc, float beta, const uint32_t *keep, float keep_scale,
                          bool bf16, hipStream_t s);

// gemm_mfma.hip -- tiled MFMA GEMMs with fused dequantisation (any accepted shape)
// Workgroups per output tile along the contraction.  An [M, NO] output with a contraction of length KC that makes
// at most 128 tiles of 128 x 128 would leave half of the 256 CUs idle: the contraction is then cut into up to 8
// runs of at least 8 stages (64 deep each), every run one workgroup, and the fp32 partial products are summed in a
// fixed order by a second kernel.  1: no split.  Depends on the shape alone.
constexpr int GEMM_SPLIT_BN = 128;
inline int gemm_splits(int M, int NO, int KC)
{
    const long tiles = (long)((M + 127) / 128) * ((NO + GEMM_SPLIT_BN - 1) / GEMM_SPLIT_BN);
    if (tiles > 128) return 1;
    const int by_cus = (int)(256 / tiles), by_depth = ((KC + 63) / 64) / 8;
    const int s = by_cus < by_depth ? by_cus : by_depth;
    return s > 8 ? 8 : (s < 1 ? 1 : s);
}
// part: gemm_splits(M, NO, KC) * M * NO floats when that count exceeds 1 (NO = N, KC = K forward; NO = K, KC = N
// backward); NULL switches splitting off
void launch_fwd_mfma(const Problem &p, const void *x, const uint32_t *packed, const void *scales,
                     const uint8_t *zeros, const void *t, const void *B, void *y, float *part, hipStream_t s);
// keep != NULL (LoRA dropout, ranks up to GEMM_MASKED_MAX_RANK): dX = dY Wd + sc keep_scale keep (.) (u A), the
// masked product added in the epilogue (the contraction is then never split)
constexpr int GEMM_MASKED_MAX_RANK = 32;
void launch_bwd_dx_mfma(const Problem &p, const void *dy, const uint32_t *packed, const void *scales,
                        const uint8_t *zeros, const void *u, const void *A, void *dx, float *part,
                        const uint32_t *keep, float keep_scale, hipStream_t s);

// gemv.hip -- small token counts: weight-streaming kernels, one pass over the packed weight
constexpr int SMALL_M_FWD_MAX = 32;   // above: the tiled GEMM with its contraction split over workgroups is faster
constexpr int SMALL_M_BWD_MAX = 32;   // backward kernel: one 16-row token block, or two where its staged form applies
constexpr int SIBLINGS_MAX_M = 16;    // sibling launches keep one token block
int gemv_bwd_slices(int N, int K, int bits);   // row slices of the backward kernel
bool fwd_small_computes_t(int rank);           // true: the forward kernel forms t = x A^T itself (unless t is handed in)
constexpr int MAX_SIBLINGS = 4;                // projections that read the same x, served by one launch
// `count` sibling projections (same x, M, K, code width, grouping, rank; own weights, adapters, N and outputs):
// y[i] (and t_out[i], if not NULL and the kernel forms t) from one launch up to 16 token rows, one launch each above;
// t_in[i] is used when the kernel does not form t (ranks above 32, or t_given: t was computed beforehand, e.g. under
// dropout).  The arrays are host arrays of `count` device pointers.  With `zpacked` (the zero-points of each
// projection in their bit-packed storage form, [N, zero_words]) `zeros` is not read; only the staged kernel for up
// to 16 rows reads that form, and where it does not take the shape nothing is launched and false comes back.
bool launch_fwd_small(const Problem &p, int count, const void *x, const uint32_t *const *packed,
                      const void *const *scales, const uint8_t *const *zeros, const void *const *A,
                      const void *const *B, const void *const *t_in, void *const *t_out, void *const *y, const int *N,
                      bool t_given, hipStream_t s, const uint32_t *const *zpacked = nullptr);
// Row slices of the backward kernel for `count` sibling projections launched together: slices[i] for each, the
// total returned (count == 1: gemv_bwd_slices).
int gemv_bwd_slices_siblings(int count, const int *N, int K, int bits, int *slices);
// dx (the sum over the siblings), dA[i], dB[i] from two launches; partial holds total_slices*M*K floats, upartial
// total_slices*1024 floats; t may be NULL if r == 0; beta != 0 accumulates into dA[i], dB[i] (beta*old + new).  The
// arrays are host arrays of `count` device pointers.  keep != NULL (LoRA dropout, single projection only): the
// adapter's share of dX is multiplied by keep_scale * keep and x stands for keep_scale * x * keep in dA.
// frozen (single projection only): the first `frozen` adapter columns have no gradient; dA is [r - frozen, K], dB
// [N, r - frozen].  zpacked: as for launch_fwd_small (here the staged kernel reads that form; false, and nothing
// launched, where it does not take the shape).
bool launch_bwd_small(const Problem &p, int count, const void *const *dy, const void *x,
                      const uint32_t *const *packed, const void *const *scales, const uint8_t *const *zeros,
                      const void *const *A, const void *const *B, const void *const *t, void *dx, float *const *dA,
                      float *const *dB, const int *N, float *partial, float *upartial, float beta, const uint32_t *keep,
                      float keep_scale, int frozen, hipStream_t s, const uint32_t *const *zpacked = nullptr);

// loss.hip -- the LREC objective (KL student || teacher + next-token CE, mean over tokens) and its gradient
// kl, ce (per token) and grad may be NULL; tok receives lambda_kl*KL + lambda_ce*CE per token, loss_mean their mean;
// grad is written multiplied by grad_scale (loss scaling)
void launch_lrec_loss(const void *student, const void *teacher, const int32_t *labels, float lambda_kl,
                      float lambda_ce, float grad_scale, float *kl, float *ce, float *tok, float *loss_mean, void *grad,
                      int M, int V, bool bf16, hipStream_t s);

}  // namespace qlora
