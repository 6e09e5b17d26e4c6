// Small token counts: the pass is bound by streaming the packed weight once from HBM (Limitations of the paper:
// the compressed weight cuts the memory traffic of both passes; this is the regime where that shows).  Launches are
// what the pass is made of at this size, so the rank-r products ride along: one launch forward, two backward
// (gemv_bwd.hip).
//
//   forward  (M <= 32)  y = x Wd^T + sc * t B^T with t = x A^T computed by the same v_mfma_f32_16x16x32 (one extra
//            fragment of A per k-step); a workgroup owns up to four blocks of 16 weight rows, its waves split K.
//            The packed words, x and A are staged through LDS by direct-to-LDS loads (gemv_fwd_m16.hpp); shapes
//            that kernel does not take stage x and A only and fetch packed words fragment-wise (gemv_fwd_impl.hpp).
//
// This file holds the host side of the forward pass; the kernels are instantiated per code width in
// gemv_fwd_b{2,3,4,8}.hip.
#include "gemv_common.hpp"

namespace qlora {

bool fwd_small_computes_t(int rank) { return rank > 0 && rank <= 32; }

bool launch_fwd_small(const Problem &p, int count, const void *x, const uint32_t *const *packed,
                      const void *const *scales, const uint8_t *const *zeros, const void *const *A,
                      const void *const *B, const void *const *t_in, void *const *t_out, void *const *y, const int *N,
                      bool t_given, hipStream_t s, const uint32_t *const *zpacked)
{
    const bool fused = fwd_small_computes_t(p.r) && !t_given;
    FwdMulti m{};
    m.count = count;
    for (int i = 0; i < count; ++i)
        m.p[i] = FwdArgs{(const uint16_t *)x,
                         packed[i],
                         (const uint16_t *)scales[i],
                         zeros[i],
                         (const uint16_t *)(A ? A[i] : nullptr),
                         (const uint16_t *)(B ? B[i] : nullptr),
                         fused ? nullptr : (const uint16_t *)(t_in ? t_in[i] : nullptr),
                         (uint16_t *)y[i],
                         fused ? (uint16_t *)(t_out ? t_out[i] : nullptr) : nullptr,
                         p.M,
                         N[i],
                         p.K,
                         p.r,
                         p.K / p.G,
                         p.sc,
                         group_magic(p.G),
                         zpacked ? zpacked[i] : nullptr,
                         zpacked ? zero_words(p.K / p.G, p.bits) : 0};
    const int rg = fused ? (p.r + 15) / 16 : 0;
    switch (p.bits) {
    case 2: return launch_fwd_small_bits<2>(m, rg, p.bf16, s);
    case 3: return launch_fwd_small_bits<3>(m, rg, p.bf16, s);
    case 4: return launch_fwd_small_bits<4>(m, rg, p.bf16, s);
    default: return launch_fwd_small_bits<8>(m, rg, p.bf16, s);
    }
}

}  // namespace qlora
