// C ABI of the library: argument validation, workspace carve-up, kernel selection.
// Nothing here touches the device before every argument has been checked.
#include "../../include/qlora.h"
#include "../../include/qlora_bench.h"
#include "kernels.hpp"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <vector>

using namespace qlora;

namespace {

constexpr size_t ALIGN = 256;

inline size_t round_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline bool misaligned(const void *p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_weight_shape(int N, int K, int bits)
{
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return QLORA_E_BITS;
    if (N < 1 || K < 1 || K % 32 != 0 || N % 8 != 0) return QLORA_E_SHAPE;
    if (K > (1 << 20) || N > (1 << 24)) return QLORA_E_SHAPE;   // kernels index groups and rows in 32 bits
    if ((long long)N * K >= (1ll << 32)) return QLORA_E_SHAPE;  // pack / unpack launch one thread per word / per code
    return QLORA_OK;
}

int check_zero_shape(int N, int groups, int bits)
{
    if (bits != 2 && bits != 3 && bits != 4 && bits != 8) return QLORA_E_BITS;
    if (N < 1 || groups < 1 || (long long)N * groups >= (1ll << 31)) return QLORA_E_SHAPE;
    return QLORA_OK;
}

int check_problem(int M, int N, int K, int bits, int G, int r, int dtype)
{
    int st = check_weight_shape(N, K, bits);
    if (st != QLORA_OK) return st;
    if (M < 1) return QLORA_E_SHAPE;
    // element indices of the activations are kept in 32 bits inside the kernels
    if ((long long)M * K >= (1ll << 31) || (long long)M * N >= (1ll << 31)) return QLORA_E_SHAPE;
    if (G < 32 || G % 32 != 0 || K % G != 0) return QLORA_E_GROUP;
    if (r < 0 || r > 64 || r % 8 != 0) return QLORA_E_RANK;
    if (dtype != QLORA_F16 && dtype != QLORA_BF16) return QLORA_E_DTYPE;
    return QLORA_OK;
}

struct Workspace {
    size_t t_off, u_off, upartial_off, partial_off, split_off, total;
    bool t_planes;      // the partial-dX region may serve as the fp32 planes of t = x A^T at small token counts: it holds
                        // at least M * K floats, the planes at most ceil(K / 128) * M * 64 of them (K >= 128: no more
                        // than that), and t is formed before anything else uses the region
};

Workspace carve(int M, int N, int K, int r, int bits)
{
    Workspace w{};
    size_t off = 0;
    w.t_off = off;
    off += round_up((size_t)M * r * 2);
    w.u_off = off;
    off += round_up((size_t)M * r * 2);
    w.upartial_off = off;
    w.partial_off = off;
    if (M <= SMALL_M_BWD_MAX) {     // the weight-streaming backward kernel: per row slice, partial u and partial dX
        off += round_up((size_t)gemv_bwd_slices(N, K, bits) * (M > 16 ? 2048 : 1024) * sizeof(float));
        w.partial_off = off;
        off += round_up((size_t)gemv_bwd_slices(N, K, bits) * M * K * sizeof(float));
    }
    w.split_off = off;              // fp32 planes of a GEMM whose contraction is split over workgroups
    const size_t sf = (size_t)gemm_splits(M, N, K), sb = (size_t)gemm_splits(M, K, N);
    const size_t pf = sf > 1 ? sf * M * N * sizeof(float) : 0, pb = sb > 1 ? sb * M * K * sizeof(float) : 0;
    off += round_up(pf > pb ? pf : pb);
    w.total = off < ALIGN ? ALIGN : off;
    w.t_planes = M <= SMALL_M_BWD_MAX && M <= LORA_DOWN_SMALL_MAX_M && K >= 128;    // (K >= 128: see Workspace)
    return w;
}

// benchmark instrumentation of the calling thread (include/qlora_bench.h); the layer's entry points only read it
thread_local hipEvent_t g_ev_before = nullptr, g_ev_after = nullptr;
thread_local int g_ev_span = 0;   // 0: events around the GEMM; 1: around the adapter kernel before it and the GEMM; 2: that kernel alone

// Tiled passes: called before the adapter kernel that precedes the GEMM (t in the forward pass, u in the backward
// pass) and between the two; the end of the GEMM is marked by GemmTimer.
inline void mark_pre_begin(hipStream_t s)
{
    if (g_ev_before && g_ev_span != 0) (void)hipEventRecord(g_ev_before, s);
}
inline void mark_pre_end(hipStream_t s)
{
    if (g_ev_after && g_ev_span == 2) (void)hipEventRecord(g_ev_after, s);
}

struct GemmTimer {   // records the two events around the scope when instrumentation is on
    hipStream_t s;
    int span;           // the spans other than 0 exist in the tiled passes only
    explicit GemmTimer(hipStream_t st, bool tiled = false) : s(st), span(tiled ? g_ev_span : 0)
    {
        if (g_ev_before && span == 0) (void)hipEventRecord(g_ev_before, s);
    }
    ~GemmTimer()
    {
        if (g_ev_after && span != 2) (void)hipEventRecord(g_ev_after, s);
    }
};

// Every entry point that launches: begin_call() after validation and before the first launch, end_call() to return.
inline void begin_call() { launch_errors_clear(); }
inline int end_call() { return launch_errors_seen() ? QLORA_E_HIP : QLORA_OK; }

}  // namespace

extern "C" {

const char *qlora_status_string(int status)
{
    switch (status) {
    case QLORA_OK: return "ok";
    case QLORA_E_NULL: return "a required pointer is NULL";
    case QLORA_E_BITS: return "bits must be 2, 3, 4 or 8";
    case QLORA_E_SHAPE: return "bad shape: need M >= 1, K % 32 == 0, N % 8 == 0 and sizes below 2^31 elements";
    case QLORA_E_GROUP: return "bad group size: need group_size % 32 == 0 and K % group_size == 0";
    case QLORA_E_RANK: return "rank must be 0 or a multiple of 8 up to 64";
    case QLORA_E_DTYPE: return "dtype must be QLORA_F16 (0) or QLORA_BF16 (1)";
    case QLORA_E_ALIGN: return "a pointer is not 16-byte aligned";
    case QLORA_E_WORKSPACE: return "workspace is NULL or smaller than qlora_workspace_bytes()";
    case QLORA_E_HIP: return "the HIP runtime reported an error";
    case QLORA_E_GIDX: return "group index out of range, or a group without exactly group_size columns";
    case QLORA_E_STATIC: return "the problem needs more scratch than the static device array holds: use qlora_linear_fwd with a workspace";
    default: return "unknown status";
    }
}

int qlora_profile_gemm(void *ev_before, void *ev_after)
{
    g_ev_before = (hipEvent_t)ev_before;
    g_ev_after = (hipEvent_t)ev_after;
    return QLORA_OK;
}

int qlora_profile_gemm_span(int span)
{
    g_ev_span = span == 1 || span == 2 ? span : 0;
    return QLORA_OK;
}

int qlora_stream_probe(const void *src, unsigned long long bytes, uint32_t *out, void *stream)
{
    if (!src || !out) return QLORA_E_NULL;
    if (misaligned(src) || misaligned(out) || bytes % 16 != 0) return QLORA_E_ALIGN;
    begin_call();
    launch_stream_probe(src, (size_t)bytes, out, (hipStream_t)stream);
    return end_call();
}

int qlora_mfma_probe(float *out, int iters, int random, void *stream)
{
    if (!out) return QLORA_E_NULL;
    if (iters < 1) return QLORA_E_SHAPE;
    if (misaligned(out)) return QLORA_E_ALIGN;
    begin_call();
    launch_mfma_probe(out, iters, random != 0, (hipStream_t)stream);
    return end_call();
}

size_t qlora_packed_words(int N, int K, int bits)
{
    if (check_weight_shape(N, K, bits) != QLORA_OK) return 0;
    return (size_t)N * ((size_t)K * bits / 32);
}

size_t qlora_workspace_bytes(int M, int N, int K, int bits, int group_size, int rank)
{
    if (check_problem(M, N, K, bits, group_size, rank, QLORA_F16) != QLORA_OK) return 0;
    return carve(M, N, K, rank, bits).total;
}

int qlora_pack(const uint8_t *codes, uint32_t *packed, int N, int K, int bits, void *stream)
{
    const int st = check_weight_shape(N, K, bits);
    if (st != QLORA_OK) return st;
    if (!codes || !packed) return QLORA_E_NULL;
    if (misaligned(codes) || misaligned(packed)) return QLORA_E_ALIGN;
    begin_call();
    launch_pack(codes, packed, N, K, bits, (hipStream_t)stream);
    return end_call();
}

int qlora_unpack(const uint32_t *packed, uint8_t *codes, int N, int K, int bits, void *stream)
{
    const int st = check_weight_shape(N, K, bits);
    if (st != QLORA_OK) return st;
    if (!codes || !packed) return QLORA_E_NULL;
    if (misaligned(codes) || misaligned(packed)) return QLORA_E_ALIGN;
    begin_call();
    launch_unpack(packed, codes, N, K, bits, (hipStream_t)stream);
    return end_call();
}

size_t qlora_packed_zero_words(int N, int groups, int bits)
{
    if (check_zero_shape(N, groups, bits) != QLORA_OK) return 0;
    return (size_t)N * (((size_t)groups * bits + 31) / 32);
}

int qlora_pack_zeros(const uint8_t *zeros, uint32_t *packed_zeros, int N, int groups, int bits, void *stream)
{
    const int st = check_zero_shape(N, groups, bits);
    if (st != QLORA_OK) return st;
    if (!zeros || !packed_zeros) return QLORA_E_NULL;
    begin_call();
    launch_pack_zeros(zeros, packed_zeros, N, groups, bits, (hipStream_t)stream);
    return end_call();
}

int qlora_unpack_zeros(const uint32_t *packed_zeros, uint8_t *zeros, int N, int groups, int bits, void *stream)
{
    const int st = check_zero_shape(N, groups, bits);
    if (st != QLORA_OK) return st;
    if (!zeros || !packed_zeros) return QLORA_E_NULL;
    begin_call();
    launch_unpack_zeros(packed_zeros, zeros, N, groups, bits, (hipStream_t)stream);
    return end_call();
}

int qlora_actorder_perm(const int32_t *g_idx, int32_t *perm, int32_t *inv_perm, int K, int group_size)
{
    if (K < 32 || K % 32 != 0 || K > (1 << 20)) return QLORA_E_SHAPE;
    if (group_size < 32 || group_size % 32 != 0 || K % group_size != 0) return QLORA_E_GROUP;
    if (!g_idx || !perm) return QLORA_E_NULL;
    const int groups = K / group_size;
    // counting sort with a fixed capacity of group_size per group: place = g * group_size + (columns of g seen so far)
    std::vector<int> seen((size_t)groups, 0);
    for (int k = 0; k < K; ++k) {
        const int g = g_idx[k];
        if (g < 0 || g >= groups || seen[(size_t)g] >= group_size) return QLORA_E_GIDX;
        ++seen[(size_t)g];
    }
    std::fill(seen.begin(), seen.end(), 0);
    for (int k = 0; k < K; ++k) {
        const int g = g_idx[k];
        const int place = g * group_size + seen[(size_t)g]++;
        perm[place] = k;
        if (inv_perm) inv_perm[k] = place;
    }
    return QLORA_OK;
}

int qlora_pack_permuted(const uint8_t *codes, const int32_t *perm, uint32_t *packed, int N, int K, int bits,
                        void *stream)
{
    const int st = check_weight_shape(N, K, bits);
    if (st != QLORA_OK) return st;
    if (!codes || !perm || !packed) return QLORA_E_NULL;
    if (misaligned(codes) || misaligned(packed)) return QLORA_E_ALIGN;
    begin_call();
    launch_pack_permuted(codes, perm, packed, N, K, bits, (hipStream_t)stream);
    return end_call();
}

int qlora_gather_columns(const void *src, const int32_t *index, void *dst, int M, int K, void *stream)
{
    if (M < 1 || K < 32 || K % 32 != 0 || K > (1 << 20) || (long)M * K >= (1L << 31)) return QLORA_E_SHAPE;
    if (!src || !index || !dst) return QLORA_E_NULL;
    if (misaligned(src) || misaligned(dst)) return QLORA_E_ALIGN;
    begin_call();
    launch_gather_columns(src, index, dst, M, K, (hipStream_t)stream);
    return end_call();
}

int qlora_linear_fwd(const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros, const void *A,
                     const void *B, void *y, void *t_save, int M, int N, int K, int bits, int group_size, int rank,
                     float alpha, int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return qlora_linear_fwd_dropout(x, packed, scales, zeros, A, B, nullptr, 1.f, y, t_save, M, N, K, bits, group_size,
                                    rank, alpha, dtype, workspace, workspace_bytes, stream);
}

// The forward pass behind every single-projection entry point.  `ws` + w.t_off holds t when it is not saved, `ws` +
// w.split_off the planes of a split contraction; ws_bytes is what the caller's buffer holds beyond `ws`.
// zpacked: the zero-points in their bit-packed storage form instead of `zeros`; a kernel that reads that form takes
// them as they are, for any other they are unpacked into zscratch (N * groups bytes) first.
static int forward(const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros, const void *A,
                   const void *B, const uint32_t *keep_mask, float keep_scale, void *y, void *t_save, int M, int N,
                   int K, int bits, int group_size, int rank, float alpha, int dtype, char *ws, const Workspace &w,
                   size_t ws_bytes, void *stream, const uint32_t *zpacked = nullptr, uint8_t *zscratch = nullptr)
{
    if (zpacked) zeros = zscratch;
    if (misaligned(zpacked)) return QLORA_E_ALIGN;
    if (!x || !packed || !scales || !zeros || !y) return QLORA_E_NULL;
    if (rank > 0 && (!A || !B)) return QLORA_E_NULL;
    if (misaligned(x) || misaligned(packed) || misaligned(scales) || misaligned(zeros) || misaligned(y) ||
        misaligned(A) || misaligned(B) || misaligned(t_save) || misaligned(ws) || misaligned(keep_mask))
        return QLORA_E_ALIGN;
    if (!ws || ws_bytes < w.total) return QLORA_E_WORKSPACE;
    if (rank == 0) keep_mask = nullptr;         // no adapter branch: nothing is dropped

    const hipStream_t s = (hipStream_t)stream;
    begin_call();
    const Problem p{M, N, K, bits, group_size, rank, rank > 0 ? alpha / (float)rank : 0.f, dtype == QLORA_BF16};
    if (M <= SMALL_M_FWD_MAX) {
        // one launch: the weight-streaming kernel also forms t (ranks up to 32, no dropout)
        void *t = rank > 0 ? (t_save ? t_save : (void *)(ws + w.t_off)) : nullptr;
        const bool t_first = rank > 0 && (keep_mask || !fwd_small_computes_t(rank));
        if (t_first)
            launch_lora_down(x, A, t, M, K, rank, p.bf16, keep_mask, keep_scale, s,
                             w.t_planes ? (float *)(ws + w.partial_off) : nullptr);
        GemmTimer timer(s);
        const void *tc = t;
        if (!zpacked || !launch_fwd_small(p, 1, x, &packed, &scales, &zeros, &A, &B, &tc, &t, &y, &N, t_first, s, &zpacked)) {
            if (zpacked) launch_unpack_zeros(zpacked, zscratch, N, K / group_size, bits, s);
            launch_fwd_small(p, 1, x, &packed, &scales, &zeros, &A, &B, &tc, &t, &y, &N, t_first, s);
        }
    } else {
        void *t = nullptr;
        mark_pre_begin(s);
        if (zpacked) launch_unpack_zeros(zpacked, zscratch, N, K / group_size, bits, s);
        if (rank > 0) {
            t = t_save ? t_save : (void *)(ws + w.t_off);
            launch_lora_down(x, A, t, M, K, rank, p.bf16, keep_mask, keep_scale, s);
        }
        mark_pre_end(s);
        GemmTimer timer(s, true);
        launch_fwd_mfma(p, x, packed, scales, zeros, t, B, y, (float *)(ws + w.split_off), s);
    }
    return end_call();
}

int qlora_linear_fwd_dropout(const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                             const void *A, const void *B, const uint32_t *keep_mask, float keep_scale, void *y,
                             void *t_save, int M, int N, int K, int bits, int group_size, int rank, float alpha,
                             int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = check_problem(M, N, K, bits, group_size, rank, dtype);
    if (st != QLORA_OK) return st;
    return forward(x, packed, scales, zeros, A, B, keep_mask, keep_scale, y, t_save, M, N, K, bits, group_size, rank,
                   alpha, dtype, (char *)workspace, carve(M, N, K, rank, bits), workspace_bytes, stream);
}

// ---- the forward pass for callers that cannot allocate: its scratch is a static device array ----------------------
namespace {

__device__ __align__(256) unsigned char scratch[QLORA_STATIC_SCRATCH_BYTES];

// Device address of this GPU's copy of `scratch` (every GPU holds its own, at its own address), looked up once per
// device.  In host code the array's name is only a handle for the runtime, never an address a kernel could use.
void *static_scratch()
{
    constexpr int MAX_DEVICES = 64;
    static std::mutex mu;
    static void *ptr[MAX_DEVICES] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> guard(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        ptr[dev] = p;
    }
    return ptr[dev];
}

// what the forward pass alone needs of a workspace: t, and the planes of a split contraction
Workspace carve_forward(int M, int N, int K, int r)
{
    Workspace w{};
    w.t_off = 0;
    w.split_off = round_up((size_t)M * r * 2);
    const size_t sf = (size_t)gemm_splits(M, N, K);
    w.total = w.split_off + (M > SMALL_M_FWD_MAX && sf > 1 ? round_up(sf * M * N * sizeof(float)) : 0);
    if (w.total < ALIGN) w.total = ALIGN;
    return w;
}

}  // namespace

int qlora_linear_fwd_static(const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                            const void *A, const void *B, void *y, void *t_save, int M, int N, int K, int bits,
                            int group_size, int rank, float alpha, int dtype, void *stream)
{
    const int st = check_problem(M, N, K, bits, group_size, rank, dtype);
    if (st != QLORA_OK) return st;
    const Workspace w = carve_forward(M, N, K, rank);
    if (w.total > (size_t)QLORA_STATIC_SCRATCH_BYTES) return QLORA_E_STATIC;   // before anything touches the device
    void *ws = static_scratch();
    if (!ws) return QLORA_E_HIP;
    return forward(x, packed, scales, zeros, A, B, nullptr, 1.f, y, t_save, M, N, K, bits, group_size, rank, alpha,
                   dtype, (char *)ws, w, (size_t)QLORA_STATIC_SCRATCH_BYTES, stream);
}

int qlora_linear_bwd(const void *dy, const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                     const void *A, const void *B, const void *t_saved, void *dx, float *dA, float *dB, int M, int N,
                     int K, int bits, int group_size, int rank, float alpha, int dtype, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    return qlora_linear_bwd_accumulate(dy, x, packed, scales, zeros, A, B, t_saved, dx, dA, dB, 0.f, M, N, K, bits,
                                       group_size, rank, alpha, dtype, workspace, workspace_bytes, stream);
}

int qlora_linear_bwd_accumulate(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                                const uint8_t *zeros, const void *A, const void *B, const void *t_saved, void *dx,
                                float *dA, float *dB, float beta, int M, int N, int K, int bits, int group_size,
                                int rank, float alpha, int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    return qlora_linear_bwd_dropout(dy, x, packed, scales, zeros, A, B, nullptr, 1.f, t_saved, dx, dA, dB, beta, M, N,
                                    K, bits, group_size, rank, alpha, dtype, workspace, workspace_bytes, stream);
}

// The backward pass behind every single-projection entry point.  frozen: leading adapter columns without gradients.
static int backward(const void *dy, const void *x, const uint32_t *packed, const void *scales, const uint8_t *zeros,
                    const void *A, const void *B, const uint32_t *keep_mask, float keep_scale, const void *t_saved,
                    void *dx, float *dA, float *dB, float beta, int frozen, int M, int N, int K, int bits,
                    int group_size, int rank, float alpha, int dtype, void *workspace, size_t workspace_bytes,
                    void *stream, const uint32_t *zpacked = nullptr, uint8_t *zscratch = nullptr)
{
    const int st = check_problem(M, N, K, bits, group_size, rank, dtype);
    if (st != QLORA_OK) return st;
    if (zpacked) zeros = zscratch;               // as in forward()
    if (misaligned(zpacked)) return QLORA_E_ALIGN;
    if (frozen < 0 || frozen % 8 != 0 || (frozen > 0 && frozen >= rank)) return QLORA_E_RANK;
    if (!dy || !packed || !scales || !zeros || !dx) return QLORA_E_NULL;
    if (rank > 0 && (!x || !A || !B || !dA || !dB)) return QLORA_E_NULL;
    if (misaligned(dy) || misaligned(x) || misaligned(packed) || misaligned(scales) || misaligned(zeros) ||
        misaligned(A) || misaligned(B) || misaligned(t_saved) || misaligned(dx) || misaligned(dA) || misaligned(dB) ||
        misaligned(workspace) || misaligned(keep_mask))
        return QLORA_E_ALIGN;
    const Workspace w = carve(M, N, K, rank, bits);
    if (!workspace || workspace_bytes < w.total) return QLORA_E_WORKSPACE;
    if (rank == 0) keep_mask = nullptr;

    const hipStream_t s = (hipStream_t)stream;
    begin_call();
    const Problem p{M, N, K, bits, group_size, rank, rank > 0 ? alpha / (float)rank : 0.f, dtype == QLORA_BF16};
    char *ws = (char *)workspace;
    bool t_ready = false, unpacked = false;
    if (M <= SMALL_M_BWD_MAX) {
        // two launches: partial dX and u over row slices of the weight, then the sums, dA and dB.  Above 16 token
        // rows only the staged kernel serves, and not every shape: then the tiled kernels below take over.
        const void *t = t_saved;
        if (rank > 0 && !t) {
            launch_lora_down(x, A, ws + w.t_off, M, K, rank, p.bf16, keep_mask, keep_scale, s,
                             w.t_planes ? (float *)(ws + w.partial_off) : nullptr);
            t = ws + w.t_off;
            t_ready = true;
        }
        bool done = false;
        {
            GemmTimer timer(s);
            float *const partial = (float *)(ws + w.partial_off), *const upartial = (float *)(ws + w.upartial_off);
            if (zpacked)
                done = launch_bwd_small(p, 1, &dy, x, &packed, &scales, &zeros, &A, &B, &t, dx, &dA, &dB, &N, partial,
                                        upartial, beta, keep_mask, keep_scale, frozen, s, &zpacked);
            if (!done) {
                if (zpacked) {
                    launch_unpack_zeros(zpacked, zscratch, N, K / group_size, bits, s);
                    unpacked = true;
                }
                done = launch_bwd_small(p, 1, &dy, x, &packed, &scales, &zeros, &A, &B, &t, dx, &dA, &dB, &N, partial,
                                        upartial, beta, keep_mask, keep_scale, frozen, s);
            }
        }
        if (done) return end_call();
    }
    void *u = nullptr;
    mark_pre_begin(s);
    if (zpacked && !unpacked) launch_unpack_zeros(zpacked, zscratch, N, K / group_size, bits, s);
    if (rank > 0) {
        u = ws + w.u_off;
        launch_lora_u(dy, B, u, M, N, rank, p.bf16, s);
    }
    mark_pre_end(s);
    {
        GemmTimer timer(s, true);
        if (keep_mask && rank > GEMM_MASKED_MAX_RANK) {
            // the GEMM leaves the base product; the adapter's masked share is added afterwards
            Problem base = p;
            base.r = 0;
            base.sc = 0.f;
            launch_bwd_dx_mfma(base, dy, packed, scales, zeros, nullptr, nullptr, dx, (float *)(ws + w.split_off), nullptr,
                               1.f, s);
        } else {                // keep_mask: the GEMM's epilogue adds the adapter's share masked per element
            launch_bwd_dx_mfma(p, dy, packed, scales, zeros, u, A, dx, (float *)(ws + w.split_off), keep_mask, keep_scale,
                               s);
        }
    }
    if (keep_mask && rank > GEMM_MASKED_MAX_RANK)
        launch_lora_dx_masked(dx, u, A, keep_mask, M, K, rank, p.sc * keep_scale, p.bf16, s);
    if (rank > 0) {
        const void *t = t_saved;
        if (!t) {
            if (!t_ready) launch_lora_down(x, A, ws + w.t_off, M, K, rank, p.bf16, keep_mask, keep_scale, s);
            t = ws + w.t_off;
        }
        launch_adapter_grads(dy, t, x, u, dB, dA, M, N, K, rank, frozen, p.sc, beta, keep_mask, keep_scale, p.bf16, s);
    }
    return end_call();
}

int qlora_linear_bwd_dropout(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                             const uint8_t *zeros, const void *A, const void *B, const uint32_t *keep_mask,
                             float keep_scale, const void *t_saved, void *dx, float *dA, float *dB, float beta, int M,
                             int N, int K, int bits, int group_size, int rank, float alpha, int dtype,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    return backward(dy, x, packed, scales, zeros, A, B, keep_mask, keep_scale, t_saved, dx, dA, dB, beta, 0, M, N, K,
                    bits, group_size, rank, alpha, dtype, workspace, workspace_bytes, stream);
}

int qlora_linear_bwd_stacked(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                             const uint8_t *zeros, const void *A, const void *B, const void *t_saved, void *dx,
                             float *dA_train, float *dB_train, float beta, int frozen_rank, int M, int N, int K,
                             int bits, int group_size, int rank, float alpha, int dtype, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    return backward(dy, x, packed, scales, zeros, A, B, nullptr, 1.f, t_saved, dx, dA_train, dB_train, beta,
                    frozen_rank, M, N, K, bits, group_size, rank, alpha, dtype, workspace, workspace_bytes, stream);
}

int qlora_linear_bwd_dropout_stacked(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                                     const uint8_t *zeros, const void *A, const void *B, const uint32_t *keep_mask,
                                     float keep_scale, const void *t_saved, void *dx, float *dA_train, float *dB_train,
                                     float beta, int frozen_rank, int M, int N, int K, int bits, int group_size,
                                     int rank, float alpha, int dtype, void *workspace, size_t workspace_bytes,
                                     void *stream)
{
    return backward(dy, x, packed, scales, zeros, A, B, keep_mask, keep_scale, t_saved, dx, dA_train, dB_train, beta,
                    frozen_rank, M, N, K, bits, group_size, rank, alpha, dtype, workspace, workspace_bytes, stream);
}

// ---- zero-points in their bit-packed storage form: the workspace is followed by room for their unpacked form
size_t qlora_workspace_bytes_zp(int M, int N, int K, int bits, int group_size, int rank)
{
    if (check_problem(M, N, K, bits, group_size, rank, QLORA_F16) != QLORA_OK) return 0;
    return carve(M, N, K, rank, bits).total + round_up((size_t)N * (K / group_size));
}

int qlora_linear_fwd_zp(const void *x, const uint32_t *packed, const void *scales, const uint32_t *packed_zeros,
                        const void *A, const void *B, void *y, void *t_save, int M, int N, int K, int bits,
                        int group_size, int rank, float alpha, int dtype, void *workspace, size_t workspace_bytes,
                        void *stream)
{
    const int st = check_problem(M, N, K, bits, group_size, rank, dtype);
    if (st != QLORA_OK) return st;
    if (!packed_zeros) return QLORA_E_NULL;
    const Workspace w = carve(M, N, K, rank, bits);
    if (!workspace || workspace_bytes < w.total + round_up((size_t)N * (K / group_size))) return QLORA_E_WORKSPACE;
    return forward(x, packed, scales, nullptr, A, B, nullptr, 1.f, y, t_save, M, N, K, bits, group_size, rank, alpha,
                   dtype, (char *)workspace, w, w.total, stream, packed_zeros, (uint8_t *)workspace + w.total);
}

int qlora_linear_bwd_zp(const void *dy, const void *x, const uint32_t *packed, const void *scales,
                        const uint32_t *packed_zeros, const void *A, const void *B, const void *t_saved, void *dx,
                        float *dA, float *dB, float beta, int M, int N, int K, int bits, int group_size, int rank,
                        float alpha, int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = check_problem(M, N, K, bits, group_size, rank, dtype);
    if (st != QLORA_OK) return st;
    if (!packed_zeros) return QLORA_E_NULL;
    const Workspace w = carve(M, N, K, rank, bits);
    if (!workspace || workspace_bytes < w.total + round_up((size_t)N * (K / group_size))) return QLORA_E_WORKSPACE;
    return backward(dy, x, packed, scales, nullptr, A, B, nullptr, 1.f, t_saved, dx, dA, dB, beta, 0, M, N, K, bits,
                    group_size, rank, alpha, dtype, workspace, w.total, stream, packed_zeros,
                    (uint8_t *)workspace + w.total);
}

namespace {

struct SiblingWorkspace {
    size_t t_off[MAX_SIBLINGS], upartial_off, partial_off, total;
};

SiblingWorkspace carve_siblings(int count, const int *N, int M, int K, int r, int bits)
{
    SiblingWorkspace w{};
    size_t off = 0;
    for (int i = 0; i < count; ++i) {
        w.t_off[i] = off;
        off += round_up((size_t)M * r * 2);
    }
    int slices[MAX_SIBLINGS];
    const size_t total_slices = (size_t)gemv_bwd_slices_siblings(count, N, K, bits, slices);
    w.upartial_off = off;
    off += round_up(total_slices * 1024 * sizeof(float));
    w.partial_off = off;
    off += round_up(total_slices * M * K * sizeof(float));
    w.total = off < ALIGN ? ALIGN : off;
    return w;
}

int check_siblings(int count, const int *N, int M, int K, int bits, int G, int r, int dtype)
{
    if (!N) return QLORA_E_NULL;
    if (count < 1 || count > QLORA_MAX_SIBLINGS || M > QLORA_SIBLINGS_MAX_M) return QLORA_E_SHAPE;
    for (int i = 0; i < count; ++i) {
        const int st = check_problem(M, N[i], K, bits, G, r, dtype);
        if (st != QLORA_OK) return st;
    }
    return QLORA_OK;
}

}  // namespace

static_assert(QLORA_MAX_SIBLINGS == MAX_SIBLINGS && QLORA_SIBLINGS_MAX_M == SIBLINGS_MAX_M, "header and kernels agree");

size_t qlora_siblings_workspace_bytes(int count, const int *N, int M, int K, int bits, int group_size, int rank)
{
    if (check_siblings(count, N, M, K, bits, group_size, rank, QLORA_F16) != QLORA_OK) return 0;
    return carve_siblings(count, N, M, K, rank, bits).total;
}

int qlora_linear_fwd_siblings(int count, const void *x, const uint32_t *const *packed, const void *const *scales,
                              const uint8_t *const *zeros, const void *const *A, const void *const *B,
                              void *const *y, void *const *t_save, const int *N, int M, int K, int bits,
                              int group_size, int rank, float alpha, int dtype, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    const int st = check_siblings(count, N, M, K, bits, group_size, rank, dtype);
    if (st != QLORA_OK) return st;
    if (!x || !packed || !scales || !zeros || !y) return QLORA_E_NULL;
    if (rank > 0 && (!A || !B)) return QLORA_E_NULL;
    if (misaligned(x) || misaligned(workspace)) return QLORA_E_ALIGN;
    for (int i = 0; i < count; ++i) {
        if (!packed[i] || !scales[i] || !zeros[i] || !y[i]) return QLORA_E_NULL;
        if (rank > 0 && (!A[i] || !B[i])) return QLORA_E_NULL;
        if (misaligned(packed[i]) || misaligned(scales[i]) || misaligned(zeros[i]) || misaligned(y[i]) ||
            (rank > 0 && (misaligned(A[i]) || misaligned(B[i]))) || (t_save && misaligned(t_save[i])))
            return QLORA_E_ALIGN;
    }
    const SiblingWorkspace w = carve_siblings(count, N, M, K, rank, bits);
    if (!workspace || workspace_bytes < w.total) return QLORA_E_WORKSPACE;

    const hipStream_t s = (hipStream_t)stream;
    begin_call();
    const Problem p{M, 0, K, bits, group_size, rank, rank > 0 ? alpha / (float)rank : 0.f, dtype == QLORA_BF16};
    char *ws = (char *)workspace;
    void *t[MAX_SIBLINGS] = {};
    const void *tc[MAX_SIBLINGS] = {};
    for (int i = 0; i < count && rank > 0; ++i) {
        t[i] = (t_save && t_save[i]) ? t_save[i] : (void *)(ws + w.t_off[i]);
        tc[i] = t[i];
        // (the partial-dX region serves as the fp32 planes of t, one projection after the other: see Workspace)
        if (!fwd_small_computes_t(rank))
            launch_lora_down(x, A[i], t[i], M, K, rank, p.bf16, nullptr, 1.f, s,
                             K >= 128 ? (float *)(ws + w.partial_off) : nullptr);
    }
    GemmTimer timer(s);
    launch_fwd_small(p, count, x, packed, scales, zeros, A, B, tc, t, y, N, false, s);
    return end_call();
}

int qlora_linear_bwd_siblings(int count, const void *const *dy, const void *x, const uint32_t *const *packed,
                              const void *const *scales, const uint8_t *const *zeros, const void *const *A,
                              const void *const *B, const void *const *t_saved, void *dx, float *const *dA,
                              float *const *dB, const int *N, int M, int K, int bits, int group_size, int rank,
                              float alpha, int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = check_siblings(count, N, M, K, bits, group_size, rank, dtype);
    if (st != QLORA_OK) return st;
    if (!dy || !packed || !scales || !zeros || !dx) return QLORA_E_NULL;
    if (rank > 0 && (!x || !A || !B || !dA || !dB)) return QLORA_E_NULL;
    if (misaligned(x) || misaligned(dx) || misaligned(workspace)) return QLORA_E_ALIGN;
    for (int i = 0; i < count; ++i) {
        if (!dy[i] || !packed[i] || !scales[i] || !zeros[i]) return QLORA_E_NULL;
        if (rank > 0 && (!A[i] || !B[i] || !dA[i] || !dB[i])) return QLORA_E_NULL;
        if (misaligned(dy[i]) || misaligned(packed[i]) || misaligned(scales[i]) || misaligned(zeros[i]) ||
            (rank > 0 && (misaligned(A[i]) || misaligned(B[i]) || misaligned(dA[i]) || misaligned(dB[i]))) ||
            (t_saved && misaligned(t_saved[i])))
            return QLORA_E_ALIGN;
    }
    const SiblingWorkspace w = carve_siblings(count, N, M, K, rank, bits);
    if (!workspace || workspace_bytes < w.total) return QLORA_E_WORKSPACE;

    const hipStream_t s = (hipStream_t)stream;
    begin_call();
    const Problem p{M, 0, K, bits, group_size, rank, rank > 0 ? alpha / (float)rank : 0.f, dtype == QLORA_BF16};
    char *ws = (char *)workspace;
    const void *t[MAX_SIBLINGS] = {};
    for (int i = 0; i < count && rank > 0; ++i) {
        t[i] = t_saved ? t_saved[i] : nullptr;
        if (!t[i]) {
            launch_lora_down(x, A[i], ws + w.t_off[i], M, K, rank, p.bf16, nullptr, 1.f, s,
                             K >= 128 ? (float *)(ws + w.partial_off) : nullptr);
            t[i] = ws + w.t_off[i];
        }
    }
    GemmTimer timer(s);
    launch_bwd_small(p, count, dy, x, packed, scales, zeros, A, B, t, dx, dA, dB, N, (float *)(ws + w.partial_off),
                     (float *)(ws + w.upartial_off), 0.f, nullptr, 1.f, 0, s);
    return end_call();
}

size_t qlora_lrec_workspace_bytes(int M)
{
    return M < 1 ? 0 : round_up((size_t)M * sizeof(float));
}

int qlora_lrec_loss(const void *student_logits, const void *teacher_logits, const int32_t *labels, float lambda_kl,
                    float lambda_ce, float *kl, float *ce, float *loss_mean, void *dlogits, int M, int V, int dtype,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    return qlora_lrec_loss_scaled(student_logits, teacher_logits, labels, lambda_kl, lambda_ce, 1.f, kl, ce, loss_mean,
                                  dlogits, M, V, dtype, workspace, workspace_bytes, stream);
}

int qlora_lrec_loss_scaled(const void *student_logits, const void *teacher_logits, const int32_t *labels,
                           float lambda_kl, float lambda_ce, float grad_scale, float *kl, float *ce, float *loss_mean,
                           void *dlogits, int M, int V, int dtype, void *workspace, size_t workspace_bytes, void *stream)
{
    if (M < 1 || V < 8 || V % 8 != 0 || (long long)M * V >= (1ll << 40)) return QLORA_E_SHAPE;
    if (dtype != QLORA_F16 && dtype != QLORA_BF16) return QLORA_E_DTYPE;
    if (!student_logits || !teacher_logits || !labels || !loss_mean) return QLORA_E_NULL;
    if (misaligned(student_logits) || misaligned(teacher_logits) || misaligned(dlogits) || misaligned(workspace) ||
        (reinterpret_cast<uintptr_t>(labels) & 3u) || (reinterpret_cast<uintptr_t>(kl) & 3u) ||
        (reinterpret_cast<uintptr_t>(ce) & 3u) || (reinterpret_cast<uintptr_t>(loss_mean) & 3u))
        return QLORA_E_ALIGN;
    if (!workspace || workspace_bytes < qlora_lrec_workspace_bytes(M)) return QLORA_E_WORKSPACE;
    begin_call();
    launch_lrec_loss(student_logits, teacher_logits, labels, lambda_kl, lambda_ce, grad_scale, kl, ce, (float *)workspace,
                     loss_mean, dlogits, M, V, dtype == QLORA_BF16, (hipStream_t)stream);
    return end_call();
}

}  // extern "C"
