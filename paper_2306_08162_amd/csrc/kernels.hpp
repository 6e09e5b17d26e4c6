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

// pack.hip
void launch_pack(const uint8_t *codes, uint32_t *packed, int N, int K, int bits, hipStream_t s);
void launch_unpack(const uint32_t *packed, uint8_t *codes, int N, int K, int bits, hipStream_t s);

// adapters.hip -- the rank-r side products and the adapter gradients
// t[M,r] = x[M,K] A[r,K]^T
void launch_lora_down(const void *x, const void *A, void *t, int M, int K, int r, bool bf16, hipStream_t s);
// u[M,r] = dy[M,N] B[N,r]; bt is scratch for B^T (N*r 16-bit values)
void launch_lora_u(const void *dy, const void *B, void *bt, void *u, int M, int N, int r, bool bf16, hipStream_t s);
// Number of token slices the adapter-gradient reductions are cut into (fixed by the shape alone).
int adapter_grad_slices(int M, int r);
// dB[N,r] = sc * dy[M,N]^T t[M,r] and dA[r,K] = sc * u[M,r]^T x[M,K], two launches for both (slice partial sums,
// then their fixed-order reduction); partial holds slices*(N+K)*r floats.
void launch_adapter_grads(const void *dy, const void *t, const void *x, const void *u, float *dB, float *dA,
                          float *partial, int M, int N, int K, int r, float sc, bool bf16, hipStream_t s);

// gemm_mfma.hip -- tiled MFMA GEMMs with fused dequantisation (any accepted shape)
void launch_fwd_mfma(const Problem &p, const void *x, const uint32_t *packed, const void *scales,
                     const uint8_t *zeros, const void *t, const void *B, void *y, hipStream_t s);
void launch_bwd_dx_mfma(const Problem &p, const void *dy, const uint32_t *packed, const void *scales,
                        const uint8_t *zeros, const void *u, const void *A, void *dx, hipStream_t s);

// gemv.hip -- small token counts: weight-streaming kernels, one pass over the packed weight
constexpr int SMALL_M_FWD_MAX = 64;   // forward kernel handles up to four 16-row token blocks
constexpr int SMALL_M_BWD_MAX = 16;   // backward kernel keeps one 16-row token block
int gemv_bwd_slices(int N, int K, int bits);   // row slices of the backward kernel
bool fwd_small_computes_t(int rank);           // true: the forward kernel forms t = x A^T itself
// y (and t_out, if not NULL and the kernel forms t) from one launch; t_in is used when the kernel does not form t
void launch_fwd_small(const Problem &p, const void *x, const uint32_t *packed, const void *scales,
                      const uint8_t *zeros, const void *A, const void *B, const void *t_in, void *t_out, void *y,
                      hipStream_t s);
// dx, dA, dB from two launches; partial holds slices*M*K floats, upartial slices*1024 floats; t may be NULL if r == 0
void launch_bwd_small(const Problem &p, const void *dy, const void *x, const uint32_t *packed, const void *scales,
                      const uint8_t *zeros, const void *A, const void *B, const void *t, void *dx, float *dA, float *dB,
                      float *partial, float *upartial, hipStream_t s);

}  // namespace qlora
