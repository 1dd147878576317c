// The register-resident matrix-vector kernel (gemv_reg_kernel.h) on plain fp16 weights (the fp16 models of Sec. 5.1):
// eligibility and launchers of the four fused one-row matvecs of the decoder layer.
#include "gemv_reg_kernel.h"

namespace relax {

// fp16 weights (a.wh): the four fused one-row matvecs of the decoder layer
bool gemv_f16w_eligible(const GemvArgs &a)
{
    const int k = a.k;
    return a.n == 1 && k >= 32 && k <= 6 * 2048 && (k % 8 == 0) && ((reinterpret_cast<uintptr_t>(a.wh) & 15) == 0) &&
           ((reinterpret_cast<uintptr_t>(a.x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(a.norm_w) & 15) == 0) && a.m >= 2;
}

bool gemv_f16w_merge_eligible(const GemvArgs &a)
{
    return a.n == 1 && a.k <= 2 * 2048 && a.k >= 32 && (a.k % 8 == 0) && a.k == a.h * a.d && (a.d % 8 == 0) && a.part != nullptr &&
           ((reinterpret_cast<uintptr_t>(a.part) & 15) == 0) && (a.part_stride % 4 == 0) && a.part_stride >= a.d / 2 + 2 &&
           a.part_splits >= 1 && a.part_splits <= kAttnMergeSplits &&
           (a.pos0 < 0 ? a.seqs.dev != nullptr : a.part_chunk > 0 && a.pos0 / a.part_chunk < a.part_splits) &&
           ((reinterpret_cast<uintptr_t>(a.wh) & 15) == 0) && a.m >= 2;
}

hipError_t launch_gemv_f16w(const GemvArgs &a, int xmode, int epi, hipStream_t stream)
{
    if (xmode == X_F16_NORM && epi == EPI_ROPE_KV) return launch_xe<X_F16_NORM, EPI_ROPE_KV, W_F16>(a, stream);
    if (xmode == X_ATTN_MERGE && epi == EPI_RESID_F32 && gemv_f16w_merge_eligible(a)) {
        GemvArgs b = a;
        b.part_used = a.pos0 >= 0 ? a.pos0 / a.part_chunk + 1 : 0;
        if (a.k <= 2048) return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 1, W_F16>(b, stream);
        return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 2, W_F16>(b, stream);
    }
    if (xmode == X_F16 && epi == EPI_RESID_F32) return launch_xe<X_F16, EPI_RESID_F32, W_F16>(a, stream);
    if (xmode == X_F32_NORM && epi == EPI_SWIGLU) return launch_xe<X_F32_NORM, EPI_SWIGLU, W_F16>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F16) return launch_xe<X_F16, EPI_RESID_F16, W_F16>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace relax
