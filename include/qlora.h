/*
 * qlora.h -- C ABI of the MI355X (gfx950) quantized LoRA linear layer.
 *
 * The layer is the one every projection of a GPTQ-quantized, LoRA-injected
 * LLaMA runs through during fine-tuning (EMEF) and error correction (LREC):
 *
 *   forward   y  = x deq(W_q)^T + (alpha/r) (x A^T) B^T            (paper Fig. 1, Sec. 3.1)
 *   backward  dX = dY deq(W_q) + (alpha/r) (dY B) A                (Sec. 3.1, "Implementation Details":
 *                                                                   the packed weight is consumed transposed,
 *                                                                   unpack + transpose + matmul in one kernel)
 *             dA = (alpha/r) (dY B)^T x,   dB = (alpha/r) dY^T (x A^T)
 *   The quantized weight is frozen: no gradient for codes, scales, zeros (Sec. 3.1).
 *
 * Symbols: M tokens, K in-features, N out-features, b bits per code,
 * G group size along K, r LoRA rank, alpha the "linear stretch" (Appendix B).
 *
 *   deq(W_q)[n,k] = s[n, k/G] * (q[n,k] - z[n, k/G])
 *
 * Storage (all row-major, dense, no strides):
 *   packed  uint32 [N, Kw], Kw = K*b/32.  Each row is a little-endian bit stream
 *           along K: code k occupies stream bits [b*k, b*k+b); stream bit p is
 *           bit (p mod 32) of word (p div 32).  b in {2,4,8}: 32/b codes per
 *           word; b = 3: codes straddle word boundaries.
 *   scales  fp16   [N, K/G]   (fp16 for both activation dtypes)
 *   zeros   uint8  [N, K/G]   zero-point as an unsigned code in [0, 2^b)
 *   x, y, dY, dX, A [r,K], B [N,r], t [M,r]: 16-bit floats of `dtype`
 *   dA [r,K], dB [N,r]: fp32
 *
 * Every pointer is a DEVICE pointer (HIP, current device) unless stated
 * otherwise; the caller owns all buffers; the library allocates nothing and
 * keeps no state between calls: the entry points are re-entrant and may be
 * called from several host threads.  Base pointers must be 16-byte aligned.
 * `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 * enqueue work on `stream` and return without synchronising.
 *
 * Errors: every function returning int returns a qlora_status_t.  Arguments
 * are validated on the host before anything is launched, so a status other
 * than QLORA_OK / QLORA_E_HIP means no device memory was written.  QLORA_E_HIP
 * reports the first failure among this call's own launches (an error some
 * earlier, unrelated HIP call left behind in the runtime is discarded first).
 *
 * Accepted domain: bits in {2,3,4,8}; K % 32 == 0, K <= 2^20; N <= 2^24;
 * N*K below 2^32 codes; M*K and M*N below 2^31 elements; group_size % 32 == 0 and
 * K % group_size == 0 (group_size == K is per-row quantisation); N % 8 == 0;
 * rank in {0, 8, 16, ..., 64}; M >= 1; dtype f16 or bf16.  rank == 0 means the
 * projection carries no adapter: A, B, t, dA, dB are ignored (may be NULL).
 */
#ifndef QLORA_H
#define QLORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { QLORA_F16 = 0, QLORA_BF16 = 1 } qlora_dtype_t;

typedef enum {
    QLORA_OK = 0,
    QLORA_E_NULL = 1,       /* a required pointer is NULL */
    QLORA_E_BITS = 2,       /* bits not in {2,3,4,8} */
    QLORA_E_SHAPE = 3,      /* M < 1, K % 32 != 0, N % 8 != 0, or a size overflows */
    QLORA_E_GROUP = 4,      /* group_size % 32 != 0 or K % group_size != 0 */
    QLORA_E_RANK = 5,       /* rank not in {0, 8, ..., 64} */
    QLORA_E_DTYPE = 6,      /* dtype not QLORA_F16 / QLORA_BF16 */
    QLORA_E_ALIGN = 7,      /* a pointer is not 16-byte aligned */
    QLORA_E_WORKSPACE = 8,  /* workspace NULL or smaller than qlora_workspace_bytes() */
    QLORA_E_HIP = 9,        /* the HIP runtime reported an error at launch */
    QLORA_E_GIDX = 10,      /* a group index is out of range, or a group does not own exactly group_size columns */
    QLORA_E_STATIC = 11     /* qlora_linear_fwd_static: the problem needs more scratch than QLORA_STATIC_SCRATCH_BYTES */
} qlora_status_t;

/* Host pointer to a static, NUL-terminated description of `status`. */
const char *qlora_status_string(int status);

/* Number of uint32 words of the packed matrix, N * K*bits/32; 0 if the arguments are invalid. */
size_t qlora_packed_words(int N, int K, int bits);

/*
 * Bytes of device scratch qlora_linear_fwd / qlora_linear_bwd need for this
 * problem (the larger of the two); 0 if the arguments are invalid.  The
 * workspace holds t = x A^T and u = dY B when they are not passed in, at up
 * to 32 token rows the per-slice partial sums of u and dX of the
 * weight-streaming backward kernels, and, for token counts whose output makes
 * too few tiles to occupy the chip, the fp32 partial products of a GEMM whose
 * contraction is split over several workgroups (all summed in a fixed order,
 * so results are bitwise reproducible run to run).
 */
size_t qlora_workspace_bytes(int M, int N, int K, int bits, int group_size, int rank);

/*
 * Bit-pack codes [N,K] (uint8, each < 2^bits) into packed [N,Kw] (layout above;
 * Sec. 3.1: the quantized weight is kept as a bit-packed INT32 matrix).
 * Done once per projection at load time.  Codes above 2^bits-1 are masked.
 */
int qlora_pack(const uint8_t *codes, uint32_t *packed, int N, int K, int bits, void *stream);

/* Inverse of qlora_pack ("standard unpacking", Sec. 3.1): packed [N,Kw] -> codes [N,K]. */
int qlora_unpack(const uint32_t *packed, uint8_t *codes, int N, int K, int bits, void *stream);

/*
 * Zero-points as quantized checkpoints store them (Sec. 2.2 / App. A: the
 * GPTQ-format files keep them bit-packed like the codes): packed_zeros
 * [N, Zw] uint32 with Zw = ceil(groups*bits/32), row n holding the zero-points
 * of its groups in order as one little-endian stream of `bits`-wide fields,
 * the last word zero-padded.  Most layer entry points take unpacked uint8
 * zero-points and these two convert at load time; qlora_linear_fwd_zp and
 * qlora_linear_bwd_zp take the packed form as it is.  groups >= 1, N >= 1,
 * N * groups < 2^31.  qlora_packed_zero_words returns N * Zw, 0 on bad arguments.
 */
size_t qlora_packed_zero_words(int N, int groups, int bits);
int qlora_pack_zeros(const uint8_t *zeros, uint32_t *packed_zeros, int N, int groups, int bits, void *stream);
int qlora_unpack_zeros(const uint32_t *packed_zeros, uint8_t *zeros, int N, int groups, int bits, void *stream);

/*
 * Checkpoints quantized in activation order (App. A: the columns are quantized
 * in order of decreasing activation size, so the G columns that share a scale
 * and zero-point are scattered over the row and the checkpoint carries a group
 * index g_idx[k] per column).  The layer entry points keep consecutive groups,
 * which is what lets one K-slice use one scale: such a checkpoint is brought
 * to that form once at load time by sorting its columns by group, and at run
 * time x is gathered into, and dX scattered out of, the sorted column order.
 * The adapter A lives in the sorted order throughout (it is trained from a
 * random start, so its column order carries no meaning); projections that read
 * the same x share one activation order and so one gather.
 *
 * qlora_actorder_perm: HOST pointers.  From g_idx [K] (each in [0, K/group_size))
 * writes perm [K], the stable sort of the columns by group (perm[j] = original
 * column that moves to place j), and, if not NULL, inv_perm [K] with
 * inv_perm[perm[j]] = j.  QLORA_E_GIDX if a group index is out of range or a
 * group does not own exactly group_size columns.  No device work.
 */
int qlora_actorder_perm(const int32_t *g_idx, int32_t *perm, int32_t *inv_perm, int K, int group_size);

/*
 * qlora_pack with a column gather: packs codes[:, perm[j]] as column j.  codes
 * [N,K] uint8, perm [K] int32, both DEVICE.  An entry of perm outside [0, K)
 * packs a zero code for that column (no out-of-bounds read).
 */
int qlora_pack_permuted(const uint8_t *codes, const int32_t *perm, uint32_t *packed, int N, int K, int bits,
                        void *stream);

/*
 * dst[m, j] = src[m, index[j]] for 16-bit elements, src and dst [M,K] row-major
 * DEVICE buffers that do not overlap, index [K] int32 DEVICE.  With index =
 * perm it brings x into the sorted column order; with index = inv_perm it
 * brings dX back to the checkpoint's.  An index outside [0, K) yields 0.
 */
int qlora_gather_columns(const void *src, const int32_t *index, void *dst, int M, int K, void *stream);

/*
 * Forward pass (Fig. 1, forward path).  Writes y [M,N] (rounded to `dtype`
 * from fp32 accumulators).  If t_save is not NULL it receives t = x A^T [M,r]
 * in `dtype` for later use by qlora_linear_bwd; otherwise t lives in the
 * workspace only.  Dequantisation is fused into the GEMM: no dequantised copy
 * of the weight is written to memory.
 */
int qlora_linear_fwd(const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                     const void *A, const void *B, void *y, void *t_save,
                     int M, int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * qlora_linear_fwd for callers that cannot allocate device memory and have no workspace to pass: code under HIP graph
 * capture, serving loops with a fixed memory plan, harnesses that forbid hipMalloc.  Same arguments and results as
 * qlora_linear_fwd without the workspace pair: the scratch the pass needs (t when it is not saved; the fp32 planes
 * of a split contraction) lives in a static device array of QLORA_STATIC_SCRATCH_BYTES inside the library, which
 * every GPU the library runs on holds until the process ends.  The call allocates and frees nothing.  Problems that
 * need more scratch are refused with QLORA_E_STATIC before anything is launched (the LLaMA-7B projections fit at
 * every token count).  Nothing in the scratch has to start at zero, and nothing is carried from call to call; but
 * all calls on one GPU share the one array, so two calls that overlap in time on the same GPU (different streams or
 * host threads) race: serialise them, or give the others a workspace through qlora_linear_fwd.  The first call on a
 * device looks the array's address up; make that call before a graph capture begins.
 */
#define QLORA_STATIC_SCRATCH_BYTES (32u << 20)
int qlora_linear_fwd_static(const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                            const void *A, const void *B, void *y, void *t_save,
                            int M, int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                            void *stream);

/*
 * Backward pass (Fig. 1, backward path; Sec. 3.1).  Writes dx [M,K] in `dtype`,
 * and, when rank > 0, dA [r,K] and dB [N,r] in fp32 (overwritten, not
 * accumulated).  t_saved is the t_save of the matching forward call, or NULL to
 * have t recomputed from x and A (what gradient checkpointing does).  x is
 * needed for dA (and for recomputing t); with rank == 0 it may be NULL.
 */
int qlora_linear_bwd(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                     const uint8_t *zeros, const void *A, const void *B, const void *t_saved,
                     void *dx, float *dA, float *dB,
                     int M, int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same with accumulation into the adapter gradients, for training steps that sum micro-batches (Appendix B:
 * a batch of 144 from micro-batches of 1, 24 or 48):  dA = beta * dA + (this call's dA), dB likewise; dx is
 * overwritten as before.  beta == 0 is qlora_linear_bwd (dA and dB are then not read).
 */
int qlora_linear_bwd_accumulate(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                                const uint8_t *zeros, const void *A, const void *B, const void *t_saved,
                                void *dx, float *dA, float *dB, float beta,
                                int M, int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * LoRA dropout (Appendix B trains with a dropout rate of 0.05).  Reading: as in the LoRA method the paper builds on,
 * dropout acts on the input of the low-rank branch only, with inverted scaling; the frozen quantized path sees x:
 *     x~ = x * keep * keep_scale,  keep_scale = 1 / (1 - p)
 *     y  = x deq(W_q)^T + (alpha/r) (x~ A^T) B^T
 *     dX = dY deq(W_q) + ((alpha/r) (dY B) A) * keep * keep_scale,   dA = (alpha/r) (dY B)^T x~,  dB unchanged in form
 * keep_mask: uint32 [M, K/32], drawn by the caller; element (m,k) is kept where bit k % 32 of word [m, k/32] is set.
 * The same mask goes to the forward and to the backward call; t_save / t_saved then hold t = x~ A^T.  keep_mask ==
 * NULL is no dropout: the calls are then qlora_linear_fwd and qlora_linear_bwd_accumulate.
 */
int qlora_linear_fwd_dropout(const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                             const void *A, const void *B, const uint32_t *keep_mask, float keep_scale,
                             void *y, void *t_save,
                             int M, int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                             void *workspace, size_t workspace_bytes, void *stream);

int qlora_linear_bwd_dropout(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                             const uint8_t *zeros, const void *A, const void *B, const uint32_t *keep_mask,
                             float keep_scale, const void *t_saved, void *dx, float *dA, float *dB, float beta,
                             int M, int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Backward pass for stacked adapters (App. D: the recovery adapter that LREC
 * trained stays on the layer, frozen, while a second pair is trained on the
 * task).  The stack is passed as one adapter of `rank` columns, A = [A_frozen;
 * A_train] [rank, K], B = [B_frozen, B_train] [N, rank], scaled by alpha / rank
 * as a whole; the forward pass is qlora_linear_fwd with that rank.  dx is the
 * gradient through the whole stack; gradients are formed for the trainable
 * pair only: dA_train [rank - frozen_rank, K], dB_train [N, rank - frozen_rank]
 * (beta as in qlora_linear_bwd_accumulate).  frozen_rank is a multiple of 8,
 * 0 <= frozen_rank < rank (0: the same as qlora_linear_bwd_accumulate), else
 * QLORA_E_RANK.  Workspace as for qlora_linear_bwd.
 */
int qlora_linear_bwd_stacked(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                             const uint8_t *zeros, const void *A, const void *B, const void *t_saved, void *dx,
                             float *dA_train, float *dB_train, float beta, int frozen_rank,
                             int M, int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * Stacked adapters trained with LoRA dropout (App. B: the fine-tuning runs use a
 * dropout rate of 0.05; App. D: the task adapter is trained on top of the frozen
 * recovery adapter): qlora_linear_bwd_stacked with the keep mask of
 * qlora_linear_bwd_dropout.  The mask acts on the input of the whole stack (both
 * pairs see keep_scale * (x . keep)), as in the forward pass
 * qlora_linear_fwd_dropout with the full rank.  keep_mask NULL: the same as
 * qlora_linear_bwd_stacked.  Arguments, layouts and errors as for the two.
 */
int qlora_linear_bwd_dropout_stacked(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                                     const uint8_t *zeros, const void *A, const void *B, const uint32_t *keep_mask,
                                     float keep_scale, const void *t_saved, void *dx, float *dA_train, float *dB_train,
                                     float beta, int frozen_rank, int M, int N, int K, int bits, int group_size,
                                     int rank, float alpha, int dtype, void *workspace, size_t workspace_bytes,
                                     void *stream);

/*
 * The layer with its zero-points left in their storage form (Sec. 3.2 counts
 * `bits` bits of zero-point per group: INT2 with G = 128 is 2 + (16 + 2) / 128
 * = 2.14 bits per weight, where a uint8 zero-point makes it 2.19).
 * packed_zeros is device memory [N, Zw] uint32 as qlora_pack_zeros writes it,
 * 16-byte aligned; everything else as for qlora_linear_fwd and
 * qlora_linear_bwd_accumulate, results bit-identical to those calls on the
 * unpacked zero-points.  The weight-streaming kernels for M <= 32 read the
 * packed rows themselves (forward: K and group_size multiples of 128, rank
 * <= 16, above 16 rows bits != 3; backward: bits != 3, above 16 rows bits
 * != 8, the column blocks of 128 or 256 dividing K and holding at most two
 * groups; both: N * groups a multiple of 16 and N * Zw of 4: the shapes of the
 * paper's models at bits 2, 4 and 8 all qualify up to 16 rows).  For
 * every other shape the zero-points are first unpacked into the workspace by
 * one more launch, which is why the workspace is larger:
 * qlora_workspace_bytes_zp = qlora_workspace_bytes plus N * groups rounded up
 * to 256 (0 on bad arguments); QLORA_E_WORKSPACE if the buffer is smaller.
 */
size_t qlora_workspace_bytes_zp(int M, int N, int K, int bits, int group_size, int rank);
int qlora_linear_fwd_zp(const void *x, const uint32_t *packed, const void *scales, const uint32_t *packed_zeros,
                        const void *A, const void *B, void *y, void *t_save, int M, int N, int K, int bits,
                        int group_size, int rank, float alpha, int dtype, void *workspace, size_t workspace_bytes,
                        void *stream);
int qlora_linear_bwd_zp(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                        const uint32_t *packed_zeros, const void *A, const void *B, const void *t_saved, void *dx,
                        float *dA, float *dB, float beta, int M, int N, int K, int bits, int group_size, int rank,
                        float alpha, int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sibling projections at small token counts.  Projections that read the same
 * input (q/k/v of an attention block, gate/up of an MLP; the paper adapts "every
 * linear projection", Appendix C) can be handed over together: one launch
 * streams all their packed weights and fetches x once per workgroup instead of
 * once per projection, and their contributions to dX are summed by the same
 * reduction that sums the row slices.  Results equal those of the per-layer
 * calls (y_i, dA_i, dB_i as above; dX = sum over i of the per-layer dX_i).
 *
 * count in [1, QLORA_MAX_SIBLINGS]; M <= QLORA_SIBLINGS_MAX_M (the
 * weight-streaming regime: larger M is what the per-layer calls are for).  The
 * siblings share M, K, bits, group_size, rank, alpha and dtype; projection i has
 * N[i] out-features and its own packed[i], scales[i], zeros[i], A[i], B[i],
 * y[i] / dy[i], dA[i], dB[i].  N and the pointer arrays are HOST arrays of `count`
 * entries (the entries are device pointers); they are read before the call
 * returns.  t_save / t_saved may be NULL, or hold NULL entries, meaning "not
 * saved" / "recompute" for that projection.  Validation and errors as above.
 */
#define QLORA_MAX_SIBLINGS 4
#define QLORA_SIBLINGS_MAX_M 16

/* Bytes of scratch the two sibling calls need (the larger of the two); 0 if the arguments are invalid. */
size_t qlora_siblings_workspace_bytes(int count, const int *N, int M, int K, int bits, int group_size, int rank);

int qlora_linear_fwd_siblings(int count, const void *x, const uint32_t *const *packed, const void *const *scales,
                              const uint8_t *const *zeros, const void *const *A, const void *const *B,
                              void *const *y, void *const *t_save, const int *N,
                              int M, int K, int bits, int group_size, int rank, float alpha, int dtype,
                              void *workspace, size_t workspace_bytes, void *stream);

int qlora_linear_bwd_siblings(int count, const void *const *dy, const void *x, const uint32_t *const *packed,
                              const void *const *scales, const uint8_t *const *zeros, const void *const *A,
                              const void *const *B, const void *const *t_saved,
                              void *dx, float *const *dA, float *const *dB, const int *N,
                              int M, int K, int bits, int group_size, int rank, float alpha, int dtype,
                              void *workspace, size_t workspace_bytes, void *stream);

/*
 * The LREC objective (Sec. 3.2 "Optimization", Eq. 1 and 2) and its gradient with respect to the student logits:
 *   per token  y_hat = softmax(student_logits[m,:]),  y = softmax(teacher_logits[m,:])
 *              KL = sum_i y_hat_i log(y_hat_i / y_i)          (student first, as Eq. 1 is written)
 *              CE = -log y_hat[labels[m]]                      (next-token cross entropy; no CE term where the label
 *                                                               is negative or not below V)
 *   *loss_mean = mean over the M tokens of lambda_kl*KL + lambda_ce*CE      (Eq. 2; factors of Appendix C)
 *   dlogits    = d loss_mean / d student_logits, in `dtype`
 * student_logits, teacher_logits, dlogits: [M,V] of `dtype` (the teacher's are its cached logits); labels int32 [M];
 * kl, ce: fp32 [M], each may be NULL; dlogits may be NULL (objective only); loss_mean: fp32 [1].  V % 8 == 0,
 * M*V below 2^40.  workspace: qlora_lrec_workspace_bytes(M) bytes.  Sums run in a fixed order: results are
 * bitwise reproducible.  Validation and errors as for the other calls.
 */
size_t qlora_lrec_workspace_bytes(int M);

int qlora_lrec_loss(const void *student_logits, const void *teacher_logits, const int32_t *labels,
                    float lambda_kl, float lambda_ce, float *kl, float *ce, float *loss_mean, void *dlogits,
                    int M, int V, int dtype, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same with loss scaling: dlogits = grad_scale * d loss_mean / d student_logits (kl, ce and loss_mean are not
 * scaled).  The mean over M tokens puts a factor 1/M on every gradient entry: at the LREC setting of Appendix C
 * (2048-token sequences, 32000 logits) most entries of an fp16 gradient would be subnormal or flush to zero;
 * a power-of-two grad_scale (undone by the caller after the backward pass, in fp32) keeps them representable.
 * grad_scale == 1 is qlora_lrec_loss.
 */
int qlora_lrec_loss_scaled(const void *student_logits, const void *teacher_logits, const int32_t *labels,
                           float lambda_kl, float lambda_ce, float grad_scale, float *kl, float *ce,
                           float *loss_mean, void *dlogits, int M, int V, int dtype,
                           void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QLORA_H */
