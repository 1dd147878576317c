// The register-resident matrix-vector kernel (gemv_reg_kernel.h) on the 4-bit stream: eligibility and launchers of every
// prologue / epilogue variant the decoder layer uses (Relax, Sec. 4.2 decode_q4 case study; Sec. 5.1 batch-1 decoding).
#include "gemv_reg_kernel.h"

namespace relax {

// rows of 16-byte packets, whole groups, at most 6 chunks of 2048 columns (the x registers of a lane)
bool gemv_reg_eligible(const GemvArgs &a)
{
    const int k = a.k;
    return k >= 32 && k <= 6 * 2048 && (k % kGroup == 0) && ((reinterpret_cast<uintptr_t>(a.q) & 15) == 0) &&
           ((reinterpret_cast<uintptr_t>(a.x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(a.norm_w) & 15) == 0) && a.m >= 2;
}

// X_ATTN_MERGE: one row, at most three chunks of columns (the split accumulators of a thread live in registers), heads
// of whole 8-element packets, 16-byte aligned partials with at most kAttnMergeSplits splits
bool gemv_merge_eligible(const GemvArgs &a)
{
    return a.n == 1 && a.k <= 3 * 2048 && a.k >= 32 && (a.k % kGroup == 0) && a.k == a.h * a.d && (a.d % 8 == 0) && a.part != nullptr &&
           ((reinterpret_cast<uintptr_t>(a.part) & 15) == 0) && (a.part_stride % 4 == 0) && a.part_stride >= a.d / 2 + 2 &&
           a.part_splits >= 1 && a.part_splits <= kAttnMergeSplits &&
           (a.pos0 < 0 ? a.seqs.dev != nullptr                       // position and split plan from the device-resident descriptor
                       : a.part_chunk > 0 && a.pos0 / a.part_chunk < a.part_splits) &&
           ((reinterpret_cast<uintptr_t>(a.q) & 15) == 0) && a.m >= 2;
}

hipError_t launch_gemv_reg(const GemvArgs &a, int xmode, int epi, hipStream_t stream)
{
    if (xmode == X_F16 && epi == EPI_F16) return launch_xe<X_F16, EPI_F16>(a, stream);
    if (xmode == X_F16_NORM && epi == EPI_ROPE_KV) return launch_xe<X_F16_NORM, EPI_ROPE_KV>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F32) return launch_xe<X_F16, EPI_RESID_F32>(a, stream);
    if (xmode == X_ATTN_MERGE && epi == EPI_RESID_F32 && gemv_merge_eligible(a)) {
        GemvArgs b = a;
        b.part_used = a.pos0 >= 0 ? a.pos0 / a.part_chunk + 1 : 0;     // splits that hold tokens (read from the descriptor when pos0 < 0)
        if (a.k <= 2048) return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 1>(b, stream);
        if (a.k > 2 * 2048) return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 3>(b, stream);
        return launch_ng<X_ATTN_MERGE, EPI_RESID_F32, 2>(b, stream);
    }
    if (xmode == X_F32_NORM && epi == EPI_SWIGLU) return launch_xe<X_F32_NORM, EPI_SWIGLU>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F16) return launch_xe<X_F16, EPI_RESID_F16>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace relax
