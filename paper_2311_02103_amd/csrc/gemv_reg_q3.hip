// The register-resident matrix-vector kernel (gemv_reg_kernel.h) on 3-bit weights in the native word layout (Sec. 5.3):
// eligibility and launchers of the fused one-row matvecs of the decoder layer and of the plain one-row matvec.
#include "gemv_reg_kernel.h"

namespace relax {

// 3-bit weights in the native word layout (a.q, a.s; group 32): the same four launches for one row of x
bool gemv_q3w_eligible(const GemvArgs &a)
{
    const int k = a.k;
    return a.n == 1 && k >= 32 && k <= 6 * 2048 && (k % 32 == 0) && ((reinterpret_cast<uintptr_t>(a.q) & 3) == 0) &&
           ((reinterpret_cast<uintptr_t>(a.x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(a.norm_w) & 15) == 0) && a.m >= 2;
}

hipError_t launch_gemv_q3w(const GemvArgs &a, int xmode, int epi, hipStream_t stream)
{
    if (xmode == X_F16 && epi == EPI_F16) return launch_xe<X_F16, EPI_F16, W_Q3>(a, stream);
    if (xmode == X_F16_NORM && epi == EPI_ROPE_KV) return launch_xe<X_F16_NORM, EPI_ROPE_KV, W_Q3>(a, stream);
    if (xmode == X_ATTN_MERGE && epi == EPI_RESID_F32 && gemv_merge_eligible(a)) {
        GemvArgs b = a;
        b.part_used = a.pos0 >= 0 ? a.pos0 / a.part_chunk + 1 : 0;
        if (a.k <= 2048) return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 1, W_Q3>(b, stream);
        if (a.k > 2 * 2048) return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 3, W_Q3>(b, stream);
        return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 2, W_Q3>(b, stream);
    }
    if (xmode == X_F16 && epi == EPI_RESID_F32) return launch_xe<X_F16, EPI_RESID_F32, W_Q3>(a, stream);
    if (xmode == X_F32_NORM && epi == EPI_SWIGLU) return launch_xe<X_F32_NORM, EPI_SWIGLU, W_Q3>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F16) return launch_xe<X_F16, EPI_RESID_F16, W_Q3>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace relax
