/*
 * CPU oracle for the quantized LoRA linear layer -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64 definition of what the layer computes, written from the paper's
 * description of the method (Sec. 3.1 "Implementation Details", Fig. 1 and
 * Appendix B "Adaptation Parameters").  It exists so that the HIP library can
 * be checked against something independent of it: it shares no source, header,
 * table or helper with the GPU code, and only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It is deliberately slow and
 * un-tuned: one loop nest per definition, no blocking, no fusion.
 *
 * Notation (paper / this file):
 *   W_q  [N,K]  integer codes q in [0, 2^b), the frozen quantized weight
 *   P    [N,Kw] the same codes bit-packed into 32-bit words, Kw = K*b/32
 *   s,z  [N,K/G] per-group scale and zero-point (group = G consecutive k)
 *   Wd   [N,K]  deq(W_q)[n,k] = s[n,k/G] * (q[n,k] - z[n,k/G])
 *   A [r,K], B [N,r]  the LoRA pair, alpha the "linear stretch"
 *   forward   y  = x Wd^T + (alpha/r) (x A^T) B^T
 *   backward  dX = dY Wd + (alpha/r) (dY B) A
 *             dB = (alpha/r) dY^T (x A^T),  dA = (alpha/r) (dY B)^T x
 *   theta_q (codes, s, z) is frozen: it gets no gradient (Sec. 3.1).
 *
 * All floating-point inputs arrive already widened, exactly, to double.
 * Parity status: every function here is pinned by tests that do not call it
 * to produce their expected value (hand-derived words, brute-force Python
 * loops, numpy float64 products, finite differences, adjoint identities).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int qo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ codes */

/*
 * Bit-packing of one weight row (Sec. 3.1, Implementation Details: the codes
 * are kept as a bit-packed INT32 matrix).  Layout: each row is a little-endian
 * bit stream along K; code k occupies stream bits [b*k, b*k+b), stream bit p
 * is bit (p mod 32) of word (p div 32).  For b in {2,4,8} this puts 32/b codes
 * in each word; for b = 3 a code may straddle two words.  Written bit by bit
 * so the layout is the definition itself.
 */
void qo_pack(const uint8_t *codes, uint32_t *P, long N, long K, int b)
{
    long Kw = K * b / 32;
    for (long n = 0; n < N; ++n) {
        uint32_t *row = P + n * Kw;
        memset(row, 0, (size_t)Kw * sizeof(uint32_t));
        for (long k = 0; k < K; ++k) {
            unsigned q = codes[n * K + k];
            for (int j = 0; j < b; ++j) {
                long p = (long)b * k + j;
                if ((q >> j) & 1u)
                    row[p >> 5] |= (uint32_t)1 << (p & 31);
            }
        }
    }
}

/* Inverse of qo_pack: read each code back bit by bit. */
void qo_unpack(const uint32_t *P, uint8_t *codes, long N, long K, int b)
{
    long Kw = K * b / 32;
    for (long n = 0; n < N; ++n) {
        const uint32_t *row = P + n * Kw;
        for (long k = 0; k < K; ++k) {
            unsigned q = 0;
            for (int j = 0; j < b; ++j) {
                long p = (long)b * k + j;
                q |= ((row[p >> 5] >> (p & 31)) & 1u) << j;
            }
            codes[n * K + k] = (uint8_t)q;
        }
    }
}

/*
 * Dequantisation, Wd[n,k] = s[n,g] * (q[n,k] - z[n,g]) with g = k / G
 * (grouped affine quantisation, Appendix B "Quantization Parameters").
 */
void qo_dequant(const uint32_t *P, const double *s, const uint8_t *z,
                double *Wd, long N, long K, int b, long G)
{
    long ng = K / G;
    uint8_t *q = (uint8_t *)malloc((size_t)K);
    for (long n = 0; n < N; ++n) {
        qo_unpack(P + n * (K * b / 32), q, 1, K, b);
        for (long k = 0; k < K; ++k) {
            long g = k / G;
            Wd[n * K + k] = s[n * ng + g] * ((double)q[k] - (double)z[n * ng + g]);
        }
    }
    free(q);
}

/* ---------------------------------------------------------------- forward */

/*
 * t = x A^T, the output of the LoRA down-projection (Fig. 1, green branch).
 * x [M,K], A [r,K], t [M,r].
 */
void qo_lora_down(const double *x, const double *A, double *t, long M, long K, long r)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        for (long j = 0; j < r; ++j) {
            double acc = 0.0;
#pragma omp simd reduction(+ : acc)
            for (long k = 0; k < K; ++k)
                acc += x[m * K + k] * A[j * K + k];
            t[m * r + j] = acc;
        }
}

/*
 * Forward pass (Fig. 1, forward path): y = x Wd^T + (alpha/r) t B^T.
 * Wd is the dequantised weight [N,K] from qo_dequant, t from qo_lora_down.
 * With r = 0 the layer is the plain quantized linear.
 */
void qo_forward(const double *x, const double *Wd, const double *t, const double *B,
                double alpha, double *y, long M, long N, long K, long r)
{
    double sc = r > 0 ? alpha / (double)r : 0.0;
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        for (long n = 0; n < N; ++n) {
            double base = 0.0;
#pragma omp simd reduction(+ : base)
            for (long k = 0; k < K; ++k)
                base += x[m * K + k] * Wd[n * K + k];
            double lora = 0.0;
            for (long j = 0; j < r; ++j)
                lora += t[m * r + j] * B[n * r + j];
            y[m * N + n] = base + sc * lora;
        }
}

/* --------------------------------------------------------------- backward */

/* u = dY B, the gradient arriving at the LoRA bottleneck. dY [M,N], B [N,r]. */
void qo_lora_u(const double *dy, const double *B, double *u, long M, long N, long r)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m)
        for (long j = 0; j < r; ++j) {
            double acc = 0.0;
            for (long n = 0; n < N; ++n)
                acc += dy[m * N + n] * B[n * r + j];
            u[m * r + j] = acc;
        }
}

/*
 * Gradient w.r.t. the layer input through the frozen quantized weight plus the
 * LoRA branch (Sec. 3.1: the backward pass uses the transposed weight):
 * dX = dY Wd + (alpha/r) u A.
 */
void qo_backward_dx(const double *dy, const double *Wd, const double *u, const double *A,
                    double alpha, double *dx, long M, long N, long K, long r)
{
    double sc = r > 0 ? alpha / (double)r : 0.0;
#pragma omp parallel for schedule(static)
    for (long m = 0; m < M; ++m) {
        double *row = dx + m * K;
        for (long k = 0; k < K; ++k)
            row[k] = 0.0;
        for (long n = 0; n < N; ++n) {
            double g = dy[m * N + n];
#pragma omp simd
            for (long k = 0; k < K; ++k)
                row[k] += g * Wd[n * K + k];
        }
        for (long j = 0; j < r; ++j) {
            double g = sc * u[m * r + j];
#pragma omp simd
            for (long k = 0; k < K; ++k)
                row[k] += g * A[j * K + k];
        }
    }
}

/*
 * Gradients of the only trainable parameters, the LoRA pair (Sec. 3.1):
 * dB[n,j] = (alpha/r) sum_m dY[m,n] t[m,j],  dA[j,k] = (alpha/r) sum_m u[m,j] x[m,k].
 */
void qo_backward_adapters(const double *dy, const double *x, const double *t, const double *u,
                          double alpha, double *dA, double *dB, long M, long N, long K, long r)
{
    double sc = r > 0 ? alpha / (double)r : 0.0;
#pragma omp parallel for schedule(static)
    for (long n = 0; n < N; ++n)
        for (long j = 0; j < r; ++j) {
            double acc = 0.0;
            for (long m = 0; m < M; ++m)
                acc += dy[m * N + n] * t[m * r + j];
            dB[n * r + j] = sc * acc;
        }
#pragma omp parallel for schedule(static)
    for (long k = 0; k < K; ++k)
        for (long j = 0; j < r; ++j) {
            double acc = 0.0;
            for (long m = 0; m < M; ++m)
                acc += u[m * r + j] * x[m * K + k];
            dA[j * K + k] = sc * acc;
        }
}
