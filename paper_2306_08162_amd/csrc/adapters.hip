// Rank-r side of the layer (Fig. 1, green LoRA branch): t = x A^T, u = dY B and the gradients of the
// only trainable parameters, dA and dB (Sec. 3.1).  All of it is HBM-bound on x / dY; fp32 accumulation,
// fixed summation order (no float atomics), so results are bitwise reproducible.
#include "common.hpp"
#include "kernels.hpp"

namespace qlora {

constexpr int ROWS_PER_WAVE = 4;

// t[m,j] = sum_k x[m,k] A[j,k].  One wave owns ROWS_PER_WAVE token rows; lanes stride along K in 16-byte
// pieces; the rank is walked 8 columns at a time so A is fetched once per row group.
template <bool BF16>
__global__ __launch_bounds__(256) void lora_down_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ A,
                                                        uint16_t *__restrict__ t, int M, int K, int r)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m0 = (blockIdx.x * 4 + wave) * ROWS_PER_WAVE;
    if (m0 >= M) return;
    for (int j0 = 0; j0 < r; j0 += 8) {
        float acc[ROWS_PER_WAVE][8];
#pragma unroll
        for (int i = 0; i < ROWS_PER_WAVE; ++i)
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) acc[i][jj] = 0.f;
        for (int k = lane * 8; k < K; k += WAVE * 8) {
            float xf[ROWS_PER_WAVE][8];
#pragma unroll
            for (int i = 0; i < ROWS_PER_WAVE; ++i) {
                const int row = min(m0 + i, M - 1);
                const u16x8_t v = *(const u16x8_t *)(x + (long)row * K + k);
#pragma unroll
                for (int e = 0; e < 8; ++e) xf[i][e] = cvt16<BF16>(v[e]);
            }
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const u16x8_t av = *(const u16x8_t *)(A + (long)(j0 + jj) * K + k);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float a = cvt16<BF16>(av[e]);
#pragma unroll
                    for (int i = 0; i < ROWS_PER_WAVE; ++i) acc[i][jj] += xf[i][e] * a;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < ROWS_PER_WAVE; ++i)
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const float v = wave_sum(acc[i][jj]);
                if (lane == 0 && m0 + i < M) t[(long)(m0 + i) * r + j0 + jj] = to16<BF16>(v);
            }
    }
}

// u[m,j] = sum_n dy[m,n] B[n,j].  Same ownership; B rows are r contiguous values, read 8 columns at a time.
template <bool BF16>
__global__ __launch_bounds__(256) void lora_u_kernel(const uint16_t *__restrict__ dy, const uint16_t *__restrict__ B,
                                                     uint16_t *__restrict__ u, int M, int N, int r)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int m0 = (blockIdx.x * 4 + wave) * ROWS_PER_WAVE;
    if (m0 >= M) return;
    for (int j0 = 0; j0 < r; j0 += 8) {
        float acc[ROWS_PER_WAVE][8];
#pragma unroll
        for (int i = 0; i < ROWS_PER_WAVE; ++i)
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) acc[i][jj] = 0.f;
        for (int n = lane * 8; n < N; n += WAVE * 8) {
            float g[ROWS_PER_WAVE][8];
#pragma unroll
            for (int i = 0; i < ROWS_PER_WAVE; ++i) {
                const int row = min(m0 + i, M - 1);
                const u16x8_t v = *(const u16x8_t *)(dy + (long)row * N + n);
#pragma unroll
                for (int e = 0; e < 8; ++e) g[i][e] = cvt16<BF16>(v[e]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const u16x8_t bv = *(const u16x8_t *)(B + (long)(n + e) * r + j0);
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) {
                    const float b = cvt16<BF16>(bv[jj]);
#pragma unroll
                    for (int i = 0; i < ROWS_PER_WAVE; ++i) acc[i][jj] += g[i][e] * b;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < ROWS_PER_WAVE; ++i)
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                const float v = wave_sum(acc[i][jj]);
                if (lane == 0 && m0 + i < M) u[(long)(m0 + i) * r + j0 + jj] = to16<BF16>(v);
            }
    }
}

// partial[slice][c][j0..j0+8) = sum over the slice's token rows of act[m,c] * side[m,j].
// A thread owns two adjacent columns c and eight rank columns; grid = (column blocks, slices, r/8).
template <bool BF16>
__global__ __launch_bounds__(256) void adapter_grad_partial_kernel(const uint16_t *__restrict__ act,
                                                                   const uint16_t *__restrict__ side,
                                                                   float *__restrict__ partial, int M, int C, int r,
                                                                   int rows_per_slice)
{
    const int c = (blockIdx.x * 256 + threadIdx.x) * 2;
    const int slice = blockIdx.y, j0 = blockIdx.z * 8;
    if (c >= C) return;
    const int m_begin = slice * rows_per_slice, m_end = min(M, m_begin + rows_per_slice);
    float acc0[8], acc1[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) acc0[jj] = acc1[jj] = 0.f;
    for (int m = m_begin; m < m_end; ++m) {
        const uint32_t pair = *(const uint32_t *)(act + (long)m * C + c);
        const float a0 = cvt16<BF16>((uint16_t)(pair & 0xffffu)), a1 = cvt16<BF16>((uint16_t)(pair >> 16));
        const u16x8_t sv = *(const u16x8_t *)(side + (long)m * r + j0);   // same address for every lane
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
            const float sj = cvt16<BF16>(sv[jj]);
            acc0[jj] += a0 * sj;
            acc1[jj] += a1 * sj;
        }
    }
    float *dst = partial + ((long)slice * C + c) * r + j0;
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
        dst[jj] = acc0[jj];
        dst[r + jj] = acc1[jj];
    }
}

// out = sc * sum over slices (in slice order) of partial; out is [C,r] or [r,C].
__global__ __launch_bounds__(256) void adapter_grad_reduce_kernel(const float *__restrict__ partial,
                                                                  float *__restrict__ out, int C, int r, int slices,
                                                                  float sc, int c_major)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)C * r) return;
    float acc = 0.f;
    for (int s = 0; s < slices; ++s) acc += partial[(long)s * C * r + idx];
    const int c = (int)(idx / r), j = (int)(idx % r);
    out[c_major ? idx : (long)j * C + c] = sc * acc;
}

void launch_lora_down(const void *x, const void *A, void *t, int M, int K, int r, bool bf16, hipStream_t s)
{
    const dim3 grid((M + 4 * ROWS_PER_WAVE - 1) / (4 * ROWS_PER_WAVE)), block(256);
    if (bf16)
        hipLaunchKernelGGL(lora_down_kernel<true>, grid, block, 0, s, (const uint16_t *)x, (const uint16_t *)A,
                           (uint16_t *)t, M, K, r);
    else
        hipLaunchKernelGGL(lora_down_kernel<false>, grid, block, 0, s, (const uint16_t *)x, (const uint16_t *)A,
                           (uint16_t *)t, M, K, r);
}

void launch_lora_u(const void *dy, const void *B, void *u, int M, int N, int r, bool bf16, hipStream_t s)
{
    const dim3 grid((M + 4 * ROWS_PER_WAVE - 1) / (4 * ROWS_PER_WAVE)), block(256);
    if (bf16)
        hipLaunchKernelGGL(lora_u_kernel<true>, grid, block, 0, s, (const uint16_t *)dy, (const uint16_t *)B,
                           (uint16_t *)u, M, N, r);
    else
        hipLaunchKernelGGL(lora_u_kernel<false>, grid, block, 0, s, (const uint16_t *)dy, (const uint16_t *)B,
                           (uint16_t *)u, M, N, r);
}

int adapter_grad_slices(int M, int C, int r)
{
    (void)C;
    if (r <= 0) return 0;
    int slices = 512 / r;                       // keeps slices * r, hence the partial buffer, bounded
    const int by_rows = (M + 31) / 32;          // at least 32 token rows per slice
    if (slices > by_rows) slices = by_rows;
    return slices < 1 ? 1 : slices;
}

void launch_adapter_grad(const void *act, const void *side, float *out, float *partial, int M, int C, int r,
                         float sc, bool c_major, bool bf16, hipStream_t s)
{
    const int slices = adapter_grad_slices(M, C, r);
    const int rows_per_slice = (M + slices - 1) / slices;
    const dim3 grid((C / 2 + 255) / 256, slices, r / 8), block(256);
    if (bf16)
        hipLaunchKernelGGL(adapter_grad_partial_kernel<true>, grid, block, 0, s, (const uint16_t *)act,
                           (const uint16_t *)side, partial, M, C, r, rows_per_slice);
    else
        hipLaunchKernelGGL(adapter_grad_partial_kernel<false>, grid, block, 0, s, (const uint16_t *)act,
                           (const uint16_t *)side, partial, M, C, r, rows_per_slice);
    const long n = (long)C * r;
    hipLaunchKernelGGL(adapter_grad_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, partial, out, C,
                       r, slices, sc, c_major ? 1 : 0);
}

}  // namespace qlora
