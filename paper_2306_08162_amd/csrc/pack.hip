// Bit-packing of the quantized weight (Sec. 3.1, "Implementation Details": the codes live in a
// bit-packed INT32 matrix) and its inverse.  Load-time work, HBM-bound, off the timed path.
#include "common.hpp"
#include "kernels.hpp"

namespace qlora {

// One thread builds one 32-bit word of the row's little-endian bit stream.
template <int BITS>
__global__ __launch_bounds__(256) void pack_kernel(const uint8_t *__restrict__ codes, uint32_t *__restrict__ packed,
                                                   int N, int K)
{
    const int Kw = K * BITS / 32;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)N * Kw) return;
    const int n = (int)(idx / Kw), w = (int)(idx % Kw);
    const uint8_t *row = codes + (long)n * K;
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int bit0 = 32 * w;
    uint32_t word = 0;
    // codes whose bit range [BITS*k, BITS*k+BITS) intersects [bit0, bit0+32)
    for (int k = bit0 / BITS; BITS * k < bit0 + 32; ++k) {
        const uint32_t q = row[k] & mask;
        const int sh = BITS * k - bit0;
        word |= sh >= 0 ? (q << sh) : (q >> (-sh));
    }
    packed[idx] = word;
}

// One thread recovers one code.
template <int BITS>
__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t *__restrict__ packed, uint8_t *__restrict__ codes,
                                                     int N, int K)
{
    const int Kw = K * BITS / 32;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)N * K) return;
    const int n = (int)(idx / K), k = (int)(idx % K);
    codes[idx] = (uint8_t)code_at<BITS>(packed + (long)n * Kw, k);
}

void launch_pack(const uint8_t *codes, uint32_t *packed, int N, int K, int bits, hipStream_t s)
{
    const long words = (long)N * (K * bits / 32);
    const dim3 grid((unsigned)((words + 255) / 256)), block(256);
    switch (bits) {
    case 2: hipLaunchKernelGGL(pack_kernel<2>, grid, block, 0, s, codes, packed, N, K); break;
    case 3: hipLaunchKernelGGL(pack_kernel<3>, grid, block, 0, s, codes, packed, N, K); break;
    case 4: hipLaunchKernelGGL(pack_kernel<4>, grid, block, 0, s, codes, packed, N, K); break;
    default: hipLaunchKernelGGL(pack_kernel<8>, grid, block, 0, s, codes, packed, N, K); break;
    }
}

void launch_unpack(const uint32_t *packed, uint8_t *codes, int N, int K, int bits, hipStream_t s)
{
    const long n = (long)N * K;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    switch (bits) {
    case 2: hipLaunchKernelGGL(unpack_kernel<2>, grid, block, 0, s, packed, codes, N, K); break;
    case 3: hipLaunchKernelGGL(unpack_kernel<3>, grid, block, 0, s, packed, codes, N, K); break;
    case 4: hipLaunchKernelGGL(unpack_kernel<4>, grid, block, 0, s, packed, codes, N, K); break;
    default: hipLaunchKernelGGL(unpack_kernel<8>, grid, block, 0, s, packed, codes, N, K); break;
    }
}

}  // namespace qlora
