// Shape-agnostic kernels: correct for every accepted shape, one output element per thread.
// They serve shapes the tiled MFMA / GEMV kernels do not cover; no attempt at speed.
#include "common.hpp"
#include "kernels.hpp"

namespace qlora {

// y[m,n] = sum_k x[m,k] s[n,g](q[n,k]-z[n,g]) + sc * sum_j t[m,j] B[n,j]      (Fig. 1, forward path)
template <int BITS, bool BF16>
__global__ __launch_bounds__(256) void fwd_generic_kernel(
    const uint16_t *__restrict__ x, const uint32_t *__restrict__ packed, const uint16_t *__restrict__ scales,
    const uint8_t *__restrict__ zeros, const uint16_t *__restrict__ t, const uint16_t *__restrict__ B,
    uint16_t *__restrict__ y, int M, int N, int K, int G, int r, float sc)
{
    const int n = blockIdx.x * 16 + (threadIdx.x & 15);
    const int m = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (m >= M || n >= N) return;
    const int ng = K / G, Kw = K * BITS / 32;
    const uint32_t *row = packed + (long)n * Kw;
    const uint16_t *xr = x + (long)m * K;
    float acc = 0.f;
    for (int g = 0; g < ng; ++g) {
        const float s = f16_bits_to_f32(scales[(long)n * ng + g]);
        const float z = (float)zeros[(long)n * ng + g];
        float part = 0.f;
        for (int k = g * G; k < (g + 1) * G; ++k)
            part += cvt16<BF16>(xr[k]) * ((float)code_at<BITS>(row, k) - z);
        acc += s * part;
    }
    float lora = 0.f;
    for (int j = 0; j < r; ++j) lora += cvt16<BF16>(t[(long)m * r + j]) * cvt16<BF16>(B[(long)n * r + j]);
    y[(long)m * N + n] = to16<BF16>(acc + sc * lora);
}

// dx[m,k] = sum_n dy[m,n] s[n,g](q[n,k]-z[n,g]) + sc * sum_j u[m,j] A[j,k]    (Sec. 3.1: transposed weight)
template <int BITS, bool BF16>
__global__ __launch_bounds__(256) void bwd_dx_generic_kernel(
    const uint16_t *__restrict__ dy, const uint32_t *__restrict__ packed, const uint16_t *__restrict__ scales,
    const uint8_t *__restrict__ zeros, const uint16_t *__restrict__ u, const uint16_t *__restrict__ A,
    uint16_t *__restrict__ dx, int M, int N, int K, int G, int r, float sc)
{
    const int k = blockIdx.x * 16 + (threadIdx.x & 15);
    const int m = blockIdx.y * 16 + (threadIdx.x >> 4);
    if (m >= M || k >= K) return;
    const int ng = K / G, Kw = K * BITS / 32, g = k / G;
    const uint16_t *dyr = dy + (long)m * N;
    float acc = 0.f;
    for (int n = 0; n < N; ++n) {
        const float s = f16_bits_to_f32(scales[(long)n * ng + g]);
        const float z = (float)zeros[(long)n * ng + g];
        acc += cvt16<BF16>(dyr[n]) * (s * ((float)code_at<BITS>(packed + (long)n * Kw, k) - z));
    }
    float lora = 0.f;
    for (int j = 0; j < r; ++j) lora += cvt16<BF16>(u[(long)m * r + j]) * cvt16<BF16>(A[(long)j * K + k]);
    dx[(long)m * K + k] = to16<BF16>(acc + sc * lora);
}

#define QLORA_DISPATCH_BITS_DTYPE(KERNEL, ...)                                                       \
    do {                                                                                             \
        if (p.bf16) {                                                                                \
            switch (p.bits) {                                                                        \
            case 2: hipLaunchKernelGGL((KERNEL<2, true>), grid, block, 0, s, __VA_ARGS__); break;    \
            case 3: hipLaunchKernelGGL((KERNEL<3, true>), grid, block, 0, s, __VA_ARGS__); break;    \
            case 4: hipLaunchKernelGGL((KERNEL<4, true>), grid, block, 0, s, __VA_ARGS__); break;    \
            default: hipLaunchKernelGGL((KERNEL<8, true>), grid, block, 0, s, __VA_ARGS__); break;   \
            }                                                                                        \
        } else {                                                                                     \
            switch (p.bits) {                                                                        \
            case 2: hipLaunchKernelGGL((KERNEL<2, false>), grid, block, 0, s, __VA_ARGS__); break;   \
            case 3: hipLaunchKernelGGL((KERNEL<3, false>), grid, block, 0, s, __VA_ARGS__); break;   \
            case 4: hipLaunchKernelGGL((KERNEL<4, false>), grid, block, 0, s, __VA_ARGS__); break;   \
            default: hipLaunchKernelGGL((KERNEL<8, false>), grid, block, 0, s, __VA_ARGS__); break;  \
            }                                                                                        \
        }                                                                                            \
    } while (0)

void launch_fwd_generic(const Problem &p, const void *x, const uint32_t *packed, const void *scales,
                        const uint8_t *zeros, const void *t, const void *B, void *y, hipStream_t s)
{
    const dim3 grid((p.N + 15) / 16, (p.M + 15) / 16), block(256);
    QLORA_DISPATCH_BITS_DTYPE(fwd_generic_kernel, (const uint16_t *)x, packed, (const uint16_t *)scales, zeros,
                              (const uint16_t *)t, (const uint16_t *)B, (uint16_t *)y, p.M, p.N, p.K, p.G, p.r, p.sc);
}

void launch_bwd_dx_generic(const Problem &p, const void *dy, const uint32_t *packed, const void *scales,
                           const uint8_t *zeros, const void *u, const void *A, void *dx, hipStream_t s)
{
    const dim3 grid((p.K + 15) / 16, (p.M + 15) / 16), block(256);
    QLORA_DISPATCH_BITS_DTYPE(bwd_dx_generic_kernel, (const uint16_t *)dy, packed, (const uint16_t *)scales, zeros,
                              (const uint16_t *)u, (const uint16_t *)A, (uint16_t *)dx, p.M, p.N, p.K, p.G, p.r, p.sc);
}

}  // namespace qlora
