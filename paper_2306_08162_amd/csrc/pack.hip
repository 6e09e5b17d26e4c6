// Bit-packing of the quantized weight (Sec. 3.1, "Implementation Details": the codes live in a
// bit-packed INT32 matrix) and its inverse.  Load-time work, HBM-bound, off the timed path.
#include "common.hpp"
#include "kernels.hpp"

#include <mutex>
#include <unordered_map>

namespace qlora {

namespace {
thread_local hipError_t first_launch_error = hipSuccess;
}

void ensure_dynamic_lds(const void *kernel, int bytes)
{
    static std::mutex mu;
    static std::unordered_map<const void *, uint64_t> done;     // kernel -> devices it has been configured on
    int dev = 0;
    (void)hipGetDevice(&dev);
    const uint64_t bit = 1ull << (dev & 63);
    std::lock_guard<std::mutex> guard(mu);
    uint64_t &mask = done[kernel];
    if (mask & bit) return;
    // remembered only when it took: a failure is reported by this call's launch and the next call tries again
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) mask |= bit;
    else if (first_launch_error == hipSuccess) first_launch_error = e;
}

void launch_errors_clear()
{
    (void)hipGetLastError();
    first_launch_error = hipSuccess;
}

void launch_errors_note()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess && first_launch_error == hipSuccess) first_launch_error = e;
}

bool launch_errors_seen() { return first_launch_error != hipSuccess; }

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

// The same with a column gather (checkpoints quantized in activation order, App. A, sorted by group at load time).
template <int BITS>
__global__ __launch_bounds__(256) void pack_permuted_kernel(const uint8_t *__restrict__ codes,
                                                            const int32_t *__restrict__ perm,
                                                            uint32_t *__restrict__ packed, int N, int K)
{
    const int Kw = K * BITS / 32;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)N * Kw) return;
    const int n = (int)(idx / Kw), w = (int)(idx % Kw);
    const uint8_t *row = codes + (long)n * K;
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int bit0 = 32 * w;
    uint32_t word = 0;
    for (int k = bit0 / BITS; BITS * k < bit0 + 32; ++k) {
        const int src = perm[k];
        const uint32_t q = (unsigned)src < (unsigned)K ? (row[src] & mask) : 0u;
        const int sh = BITS * k - bit0;
        word |= sh >= 0 ? (q << sh) : (q >> (-sh));
    }
    packed[idx] = word;
}

// Column gather of a 16-bit matrix.  A workgroup copies GATHER_ROWS whole rows into LDS with row-contiguous 16-byte
// loads (scattered 2-byte reads from global memory move a fraction of what contiguous requests do), then every thread
// builds eight neighbouring output columns per row from LDS and writes them with one 16-byte store.  The index is read
// once per thread and row block.  A workgroup takes as many rows as fit GATHER_LDS_BYTES (at most GATHER_ROWS); rows
// longer than that take the direct kernel below.
constexpr int GATHER_ROWS = 2;
constexpr int GATHER_LDS_BYTES = 16384;
constexpr int GATHER_LDS_K = 32768;      // one row of 64 KB: the most a launch gets without asking for more
__global__ __launch_bounds__(256) void gather_columns_lds_kernel(const uint16_t *__restrict__ src,
                                                                 const int32_t *__restrict__ index,
                                                                 uint16_t *__restrict__ dst, int M, int K, int R)
{
    extern __shared__ uint16_t rows[];   // R x K
    const int m0 = blockIdx.x * R;
    const int nrows = m0 + R <= M ? R : M - m0;
    const int pieces = nrows * (K / 8);                        // the rows are adjacent in memory: one flat copy
    const u32x4_t *from = reinterpret_cast<const u32x4_t *>(src + (long)m0 * K);
    for (int p = threadIdx.x; p < pieces; p += 256) reinterpret_cast<u32x4_t *>(rows)[p] = from[p];
    __syncthreads();
    for (int j0 = threadIdx.x * 8; j0 < K; j0 += 256 * 8) {
        int col[8];
        bool ok[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int v = index[j0 + e];
            ok[e] = (unsigned)v < (unsigned)K;
            col[e] = ok[e] ? v : 0;
        }
        for (int i = 0; i < nrows; ++i) {
            const uint16_t *row = rows + i * K;
            uint16_t v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = ok[e] ? row[col[e]] : (uint16_t)0;
            u32x4_t out;
            out[0] = v[0] | ((uint32_t)v[1] << 16);
            out[1] = v[2] | ((uint32_t)v[3] << 16);
            out[2] = v[4] | ((uint32_t)v[5] << 16);
            out[3] = v[6] | ((uint32_t)v[7] << 16);
            *reinterpret_cast<u32x4_t *>(dst + (long)(m0 + i) * K + j0) = out;
        }
    }
}

// The same without LDS, for rows too long to stage: a thread owns eight neighbouring output columns and walks
// GATHER_ROWS rows with the same eight source columns.
__global__ __launch_bounds__(256) void gather_columns_kernel(const uint16_t *__restrict__ src,
                                                             const int32_t *__restrict__ index,
                                                             uint16_t *__restrict__ dst, int M, int K)
{
    const int j0 = (blockIdx.y * 256 + threadIdx.x) * 8;
    if (j0 >= K) return;
    int from[8];
    bool ok[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int v = index[j0 + e];
        ok[e] = (unsigned)v < (unsigned)K;
        from[e] = ok[e] ? v : 0;
    }
    const int m0 = blockIdx.x * GATHER_ROWS;
    const int m1 = m0 + GATHER_ROWS < M ? m0 + GATHER_ROWS : M;
    for (int m = m0; m < m1; ++m) {
        const uint16_t *row = src + (long)m * K;
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = ok[e] ? row[from[e]] : (uint16_t)0;
        u32x4_t out;
        out[0] = v[0] | ((uint32_t)v[1] << 16);
        out[1] = v[2] | ((uint32_t)v[3] << 16);
        out[2] = v[4] | ((uint32_t)v[5] << 16);
        out[3] = v[6] | ((uint32_t)v[7] << 16);
        *reinterpret_cast<u32x4_t *>(dst + (long)m * K + j0) = out;
    }
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

// Zero-points as checkpoints store them: BITS wide, bit-packed per weight row in group order (the codes' stream
// convention), each row rounded up to whole words.  One thread builds one word / recovers one zero-point.
template <int BITS>
__global__ __launch_bounds__(256) void pack_zeros_kernel(const uint8_t *__restrict__ zeros, uint32_t *__restrict__ packed,
                                                         int N, int groups, int zw)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)N * zw) return;
    const int n = (int)(idx / zw), w = (int)(idx % zw);
    const uint8_t *row = zeros + (long)n * groups;
    constexpr uint32_t mask = (1u << BITS) - 1u;
    const int bit0 = 32 * w;
    uint32_t word = 0;
    for (int g = bit0 / BITS; BITS * g < bit0 + 32 && g < groups; ++g) {
        const uint32_t q = row[g] & mask;
        const int sh = BITS * g - bit0;
        word |= sh >= 0 ? (q << sh) : (q >> (-sh));
    }
    packed[idx] = word;
}

template <int BITS>
__global__ __launch_bounds__(256) void unpack_zeros_kernel(const uint32_t *__restrict__ packed, uint8_t *__restrict__ zeros,
                                                           int N, int groups, int zw)
{
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long)N * groups) return;
    const int n = (int)(idx / groups), g = (int)(idx % groups);
    zeros[idx] = (uint8_t)code_at<BITS>(packed + (long)n * zw, g);   // a straddling field ends inside the padded row
}

void launch_pack(const uint8_t *codes, uint32_t *packed, int N, int K, int bits, hipStream_t s)
{
    const long words = (long)N * (K * bits / 32);
    const dim3 grid((unsigned)((words + 255) / 256)), block(256);
    switch (bits) {
    case 2: QLORA_LAUNCH(pack_kernel<2>, grid, block, 0, s, codes, packed, N, K); break;
    case 3: QLORA_LAUNCH(pack_kernel<3>, grid, block, 0, s, codes, packed, N, K); break;
    case 4: QLORA_LAUNCH(pack_kernel<4>, grid, block, 0, s, codes, packed, N, K); break;
    default: QLORA_LAUNCH(pack_kernel<8>, grid, block, 0, s, codes, packed, N, K); break;
    }
}

void launch_pack_permuted(const uint8_t *codes, const int32_t *perm, uint32_t *packed, int N, int K, int bits,
                          hipStream_t s)
{
    const long words = (long)N * (K * bits / 32);
    const dim3 grid((unsigned)((words + 255) / 256)), block(256);
    switch (bits) {
    case 2: QLORA_LAUNCH(pack_permuted_kernel<2>, grid, block, 0, s, codes, perm, packed, N, K); break;
    case 3: QLORA_LAUNCH(pack_permuted_kernel<3>, grid, block, 0, s, codes, perm, packed, N, K); break;
    case 4: QLORA_LAUNCH(pack_permuted_kernel<4>, grid, block, 0, s, codes, perm, packed, N, K); break;
    default: QLORA_LAUNCH(pack_permuted_kernel<8>, grid, block, 0, s, codes, perm, packed, N, K); break;
    }
}

void launch_gather_columns(const void *src, const int32_t *index, void *dst, int M, int K, hipStream_t s)
{
    if (K <= GATHER_LDS_K) {
        int R = GATHER_LDS_BYTES / (K * 2);
        R = R < 1 ? 1 : (R > GATHER_ROWS ? GATHER_ROWS : R);
        QLORA_LAUNCH(gather_columns_lds_kernel, dim3((unsigned)((M + R - 1) / R)), dim3(256), (size_t)R * K * 2, s,
                           (const uint16_t *)src, index, (uint16_t *)dst, M, K, R);
        return;
    }
    const unsigned row_blocks = (unsigned)((M + GATHER_ROWS - 1) / GATHER_ROWS);
    const dim3 grid(row_blocks, (unsigned)((K / 8 + 255) / 256)), block(256);
    QLORA_LAUNCH(gather_columns_kernel, grid, block, 0, s, (const uint16_t *)src, index, (uint16_t *)dst, M, K);
}

void launch_unpack(const uint32_t *packed, uint8_t *codes, int N, int K, int bits, hipStream_t s)
{
    const long n = (long)N * K;
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    switch (bits) {
    case 2: QLORA_LAUNCH(unpack_kernel<2>, grid, block, 0, s, packed, codes, N, K); break;
    case 3: QLORA_LAUNCH(unpack_kernel<3>, grid, block, 0, s, packed, codes, N, K); break;
    case 4: QLORA_LAUNCH(unpack_kernel<4>, grid, block, 0, s, packed, codes, N, K); break;
    default: QLORA_LAUNCH(unpack_kernel<8>, grid, block, 0, s, packed, codes, N, K); break;
    }
}

void launch_pack_zeros(const uint8_t *zeros, uint32_t *packed, int N, int groups, int bits, hipStream_t s)
{
    const int zw = (groups * bits + 31) / 32;
    const dim3 grid((unsigned)(((long)N * zw + 255) / 256)), block(256);
    switch (bits) {
    case 2: QLORA_LAUNCH(pack_zeros_kernel<2>, grid, block, 0, s, zeros, packed, N, groups, zw); break;
    case 3: QLORA_LAUNCH(pack_zeros_kernel<3>, grid, block, 0, s, zeros, packed, N, groups, zw); break;
    case 4: QLORA_LAUNCH(pack_zeros_kernel<4>, grid, block, 0, s, zeros, packed, N, groups, zw); break;
    default: QLORA_LAUNCH(pack_zeros_kernel<8>, grid, block, 0, s, zeros, packed, N, groups, zw); break;
    }
}

void launch_unpack_zeros(const uint32_t *packed, uint8_t *zeros, int N, int groups, int bits, hipStream_t s)
{
    const int zw = (groups * bits + 31) / 32;
    const dim3 grid((unsigned)(((long)N * groups + 255) / 256)), block(256);
    switch (bits) {
    case 2: QLORA_LAUNCH(unpack_zeros_kernel<2>, grid, block, 0, s, packed, zeros, N, groups, zw); break;
    case 3: QLORA_LAUNCH(unpack_zeros_kernel<3>, grid, block, 0, s, packed, zeros, N, groups, zw); break;
    case 4: QLORA_LAUNCH(unpack_zeros_kernel<4>, grid, block, 0, s, packed, zeros, N, groups, zw); break;
    default: QLORA_LAUNCH(unpack_zeros_kernel<8>, grid, block, 0, s, packed, zeros, N, groups, zw); break;
    }
}

// ---- stream probe (benchmark instrumentation): reads a buffer once and does nothing else
constexpr int PROBE_WGS = 1024, PROBE_THREADS = 256;

__global__ __launch_bounds__(PROBE_THREADS) void stream_probe_kernel(const u32x4_t *__restrict__ src, long pieces,
                                                                     uint32_t *__restrict__ part)
{
    __shared__ uint32_t red[PROBE_THREADS / WAVE];
    const long step = (long)PROBE_WGS * PROBE_THREADS;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    long i = (long)blockIdx.x * PROBE_THREADS + threadIdx.x;
    for (; i + 3 * step < pieces; i += 4 * step) {          // four loads in flight per thread
        const u32x4_t a = src[i], b = src[i + step], c = src[i + 2 * step], d = src[i + 3 * step];
        acc ^= a ^ b ^ c ^ d;
    }
    for (; i < pieces; i += step) acc ^= src[i];
    uint32_t v = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v ^= (uint32_t)__shfl_xor((int)v, off, WAVE);
    if ((threadIdx.x & (WAVE - 1)) == 0) red[threadIdx.x / WAVE] = v;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

void launch_stream_probe(const void *src, size_t bytes, uint32_t *out, hipStream_t s)
{
    static_assert(PROBE_WGS == 1024, "the header promises 1024 partial words");
    QLORA_LAUNCH(stream_probe_kernel, dim3(PROBE_WGS), dim3(PROBE_THREADS), 0, s, (const u32x4_t *)src,
                 (long)(bytes / 16), out);
}

// ---- matrix-core probe (benchmark instrumentation): register-resident MFMAs and nothing else
constexpr int MFMA_PROBE_WGS = 256, MFMA_PROBE_THREADS = 512;

__device__ __forceinline__ uint32_t probe_mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

template <bool RANDOM>
__global__ __launch_bounds__(MFMA_PROBE_THREADS) void mfma_probe_kernel(float *__restrict__ out, int iters)
{
    float16_t acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    half8_t a[4], b[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (RANDOM) {
                const uint32_t r = probe_mix(threadIdx.x * 64 + s * 8 + i + blockIdx.x * 7919);
                a[s][i] = (half_t)((float)((int)(r & 0xffffu) - 32768) * (1.f / 32768.f));
                b[s][i] = (half_t)((float)((int)(r >> 16) - 32768) * (1.f / 32768.f));
            } else {
                a[s][i] = (half_t)(float)(threadIdx.x & 3);
                b[s][i] = (half_t)1.f;
            }
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i & 3], b[(i + (i >> 2)) & 3], acc[i], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[i][v];
    out[blockIdx.x * MFMA_PROBE_THREADS + threadIdx.x] = sum;
}

void launch_mfma_probe(float *out, int iters, bool random, hipStream_t s)
{
    if (random) QLORA_LAUNCH(mfma_probe_kernel<true>, dim3(MFMA_PROBE_WGS), dim3(MFMA_PROBE_THREADS), 0, s, out, iters);
    else QLORA_LAUNCH(mfma_probe_kernel<false>, dim3(MFMA_PROBE_WGS), dim3(MFMA_PROBE_THREADS), 0, s, out, iters);
}

}  // namespace qlora
