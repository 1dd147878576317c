// Internal definitions shared by the HIP translation units of librelax_mi355.so.
// Not part of the C ABI (include/relax_mi355.h is).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "relax_mi355.h"

namespace relax {

#if defined(__HIPCC__)
// A load of data that this launch touches once (a weight stream, the KV cache of a decode row): the non-temporal hint keeps
// it from displacing what the caches hold for re-use.  Measured on the 7B decode layer: 45.1 -> 41.7 us per layer call with
// the hint on the weight loads of the matvec kernel and the K / V loads of the split attention kernel.
template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
    return __builtin_nontemporal_load(p);
}
__device__ __forceinline__ uint4 stream_load(const uint4 *p)      // HIP's uint4 is a struct: go through the native vector type
{
    typedef uint32_t native4 __attribute__((ext_vector_type(4)));
    const native4 v = __builtin_nontemporal_load(reinterpret_cast<const native4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
#endif


constexpr int kWave = 64;            // CDNA wavefront
constexpr int kGroup = 32;           // sub-group the kernels walk in: 32 columns = four packed words.  The quantisation group of a matrix
                                     // is 32, 64 or 128 columns: 1, 2 or 4 neighbouring sub-groups share one scale (gshift = 0, 1, 2)
constexpr int kMaxK = 28672;         // x row (fp16) + per-group terms must fit 64 KB of LDS
constexpr int kInlineSeqs = 16;      // ragged descriptors up to this many sequences ride in kernel arguments

// The ragged batch as the kernels see it.  The symbolic values (n, B, every L_b) are plain
// kernel arguments (Sec. 3.3: symbolic values travel as extra scalar arguments); a batch
// with more than kInlineSeqs sequences is copied to a device table in the workspace, the
// device-side analogue of the runtime shape heap of Sec. 4.7.
struct SeqTable {
    int32_t B;
    int32_t n;
    int32_t q_max;                   // longest q_len of the call (host-side dispatch: decode vs prefill attention)
    const int32_t *dev;              // [4][B]: q_start, q_len, kv_len, slot; nullptr -> inline arrays
    int32_t q_start[kInlineSeqs];
    int32_t q_len[kInlineSeqs];
    int32_t kv_len[kInlineSeqs];
    int32_t slot[kInlineSeqs];
};

struct RowInfo {
    int32_t seq, pos, slot;
};

// The only row of a call whose descriptor the host holds: its position and slot travel as two scalars, and the kernel
// has them with its first round of argument loads instead of reading the table.  pos < 0: resolve on the device.
struct HostRow {
    int32_t pos, slot;
};
inline HostRow host_row(const SeqTable &st)
{
    if (st.n == 1 && st.B == 1 && st.dev == nullptr) return {st.kv_len[0] - st.q_len[0] - st.q_start[0], st.slot[0]};
    return {-1, 0};
}

// row of the call -> (sequence, position in its cache slot, slot)
__device__ inline RowInfo row_info(const SeqTable &st, int32_t row)
{
    RowInfo r;
    if (st.B == 1 && !st.dev) {                                // one sequence (batch-1 decode, a single prefill): no walk
        r.seq = 0;
        r.pos = st.kv_len[0] - st.q_len[0] + (row - st.q_start[0]);
        r.slot = st.slot[0];
    } else if (st.q_max == 1 && st.n == st.B) {
        // a decode batch (every sequence brings one row, so row b is sequence b): no walk over the starts -- one read of
        // the device table, or one pass of compares over the inline one instead of the cumulative search below
        r.seq = row;
        if (st.dev) {
            r.pos = st.dev[2 * st.B + row] - 1;
            r.slot = st.dev[3 * st.B + row];
        } else {
            int kl = st.kv_len[0], sl = st.slot[0];
#pragma unroll
            for (int j = 1; j < kInlineSeqs; ++j) {
                kl = row == j ? st.kv_len[j] : kl;
                sl = row == j ? st.slot[j] : sl;
            }
            r.pos = kl - 1;
            r.slot = sl;
        }
    } else if (st.dev) {
        const int32_t *qs = st.dev, *ql = st.dev + st.B, *kl = st.dev + 2 * st.B, *sl = st.dev + 3 * st.B;
        int b = 0;
        while (b + 1 < st.B && row >= qs[b] + ql[b]) ++b;
        r.seq = b;
        r.pos = kl[b] - ql[b] + (row - qs[b]);
        r.slot = sl[b];
    } else {
        // static indices only: a dynamic index into the by-value table would go through a flat load of the kernel
        // arguments, and a flat load in flight turns every later wait of the kernel into a wait for all loads
        int b = 0, qs = st.q_start[0], ql = st.q_len[0], kl = st.kv_len[0], sl = st.slot[0];
#pragma unroll
        for (int j = 0; j < kInlineSeqs - 1; ++j) {
            const bool adv = j + 1 < st.B && row >= st.q_start[j] + st.q_len[j];
            b = adv ? j + 1 : b;
            qs = adv ? st.q_start[j + 1] : qs;
            ql = adv ? st.q_len[j + 1] : ql;
            kl = adv ? st.kv_len[j + 1] : kl;
            sl = adv ? st.slot[j + 1] : sl;
        }
        r.seq = b;
        r.pos = kl - ql + (row - qs);
        r.slot = sl;
    }
    return r;
}

// ---- wavefront reductions without the LDS crossbar ------------------------------------------------------------------
// The exchange with lane ^ 32 and lane ^ 16 is one v_permlane32_swap / v_permlane16_swap (two copies of v in, the lower /
// even and the upper / odd quarter-rows out), the one with lane ^ 8 .. lane ^ 1 a DPP row rotation or quad permutation:
// register-to-register moves of a few cycles each, where a ds_bpermute costs a trip through the LDS and a wait.  The
// partners are those of a butterfly over lane ^ 32, 16, 8, 4, 2, 1 in this order (after the step for ^ 8 the lanes i and
// i ^ 8 hold the same value, so the rotation by 4 hands lane i what lane i ^ 4 holds), hence every lane ends with the
// same bits as that butterfly gives.
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
template <int CTRL>
__device__ __forceinline__ float lane_dpp(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// (v[lane & 31], v[lane | 32]): both halves of the pair (lane, lane ^ 32), the same in both lanes of the pair
__device__ __forceinline__ float2 pair_xor32(float v)
{
    const unsigned int u = __builtin_bit_cast(unsigned int, v);
    const u32x2_t r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned int lo = r.x, hi = r.y;    // element copies: a bit_cast applied to the subscript itself reads word 0
    return make_float2(__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi));
}
// the same for the pair (lane, lane ^ 16)
__device__ __forceinline__ float2 pair_xor16(float v)
{
    const unsigned int u = __builtin_bit_cast(unsigned int, v);
    const u32x2_t r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const unsigned int lo = r.x, hi = r.y;    // element copies: a bit_cast applied to the subscript itself reads word 0
    return make_float2(__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi));
}
__device__ __forceinline__ float xor32_sum(float v) { const float2 p = pair_xor32(v); return p.x + p.y; }
__device__ __forceinline__ float xor16_sum(float v) { const float2 p = pair_xor16(v); return p.x + p.y; }

// the value lane ^ OFF holds, for OFF < 16 (DPP only; lane ^ 4 = mirror of the half row of eight, then of the quad)
template <int OFF>
__device__ __forceinline__ float lane_xor(float v)
{
    static_assert(OFF == 1 || OFF == 2 || OFF == 4 || OFF == 8, "within a row of 16 lanes");
    if (OFF == 1) return lane_dpp<0xB1>(v);
    if (OFF == 2) return lane_dpp<0x4E>(v);
    if (OFF == 4) return lane_dpp<0x1B>(lane_dpp<0x141>(v));
    return lane_dpp<0x128>(v);
}
// v + (the value lane ^ OFF holds), any OFF of a wavefront
template <int OFF>
__device__ __forceinline__ float lane_xor_sum(float v)
{
    if constexpr (OFF == 32) return xor32_sum(v);
    else if constexpr (OFF == 16) return xor16_sum(v);
    else return v + lane_xor<OFF>(v);
}

// V partial sums per lane -> lane l holds the total of value l % V (a transposing reduction: the number of live values
// halves with every exchange)
template <int V, int BIT = 1>
__device__ __forceinline__ void fold_values(float *v, int lane)
{
    if constexpr (BIT < V) {
        const bool up = lane & BIT;
#pragma unroll
        for (int i = 0; i < V / (2 * BIT); ++i) {
            const float keep = up ? v[2 * i + 1] : v[2 * i], give = up ? v[2 * i] : v[2 * i + 1];
            v[i] = keep + lane_xor<BIT>(give);
        }
        fold_values<V, 2 * BIT>(v, lane);
    }
}
// the rest of the sum over the wavefront once the values are folded.  The step over the quads of a row is a rotation by
// four lanes, not lane ^ 4 (the rotation by eight that follows completes the row either way): the same instructions, in
// the same order, as the one- and two-value reductions of the matvec kernels, so a row's sum has the same bits whether
// it was reduced alone or next to the sums of other rows.
template <int OFF>
__device__ __forceinline__ float sum_from(float r)
{
    if constexpr (OFF == 4) return sum_from<8>(r + lane_dpp<0x124>(r));
    else if constexpr (OFF < kWave) return sum_from<2 * OFF>(lane_xor_sum<OFF>(r));
    else return r;
}
// register-to-register exchanges only (DPP, permlane swaps)
template <int V>
__device__ __forceinline__ float reduce_many(float *v, int lane)
{
    static_assert(V == 1 || V == 2 || V == 4 || V == 8, "1, 2, 4 or 8 values");
    fold_values<V>(v, lane);
    return sum_from<V>(v[0]);
}

__device__ inline float wave_sum(float v)
{
    v = xor32_sum(v);
    v = xor16_sum(v);
    v += lane_dpp<0x128>(v);                  // row_ror:8 = lane ^ 8
    v += lane_dpp<0x124>(v);                  // row_ror:4: the value lane ^ 4 holds
    v += lane_dpp<0x4E>(v);                   // quad_perm [2,3,0,1] = lane ^ 2
    v += lane_dpp<0xB1>(v);                   // quad_perm [1,0,3,2] = lane ^ 1
    return v;
}

__device__ inline float wave_max(float v)
{
    float2 p = pair_xor32(v);
    v = fmaxf(p.x, p.y);
    p = pair_xor16(v);
    v = fmaxf(p.x, p.y);
    v = fmaxf(v, lane_dpp<0x128>(v));
    v = fmaxf(v, lane_dpp<0x124>(v));
    v = fmaxf(v, lane_dpp<0x4E>(v));
    v = fmaxf(v, lane_dpp<0xB1>(v));
    return v;
}

// 1 / sqrt(mean square + eps) of an RMSNorm from the sum of squares: one multiply-add and v_rsq_f32 (1 ulp) behind the
// reduction instead of two IEEE divisions and a square root (some forty dependent instructions that every fused
// prologue waits for); 1 / k does not depend on the data and can be ready before the sum is.  Every kernel that
// normalises uses this, so the fused and the stand-alone forms still agree bit for bit.
__device__ __forceinline__ float rms_scale(float sum_sq, float inv_k, float eps) { return __builtin_amdgcn_rsqf(fmaf(sum_sq, inv_k, eps)); }

__device__ inline float h2f(uint16_t bits) { return __half2float(__ushort_as_half(bits)); }
__device__ inline uint16_t f2h(float v) { return __half_as_ushort(__float2half_rn(v)); }

// Decode of one stored code: nibble e of a word -> integer in -8..7 (offset-binary).
__device__ inline int decode_code(uint32_t word, int e) { return (int)((word >> (4 * e)) & 0xFu) - 8; }

inline int groups_of(int k) { return (k + kGroup - 1) / kGroup; }
// quantisation group of a matrix descriptor (0 reads as 32) -> shift from sub-group index to scale index; -1: unsupported
inline int gshift_of(int group) { return (group == 0 || group == 32) ? 0 : group == 64 ? 1 : group == 128 ? 2 : -1; }
// scales per row: one per (32 << gshift) columns, the last group short when that does not divide k
__host__ __device__ inline int scales_per_row(int k, int gshift) { return (k + (kGroup << gshift) - 1) >> (5 + gshift); }   // kGroup = 32: a shift, not a division (these run ahead of a kernel's first load)

// ---- launchers (defined in the .hip files), all asynchronous on `stream` --------------------------------------

enum XMode { X_F16 = 0, X_F16_NORM = 1, X_F32_NORM = 2, X_ATTN_MERGE = 3 };
constexpr int kAttnMergeSplits = 8;  // splits along L that the matvec prologue of X_ATTN_MERGE folds (one round of loads)
// Split plan of the folded form for one decode row with L cached tokens: at most max_splits chunks of whole wavefront steps
// (32 tokens), none shorter than 64 tokens unless L is.  The host evaluates it when it knows L; with a device-resident
// descriptor both kernels evaluate it from the L they read (the launch then always has max_splits slices).
// x / d for the few divisors a split count takes: constant divisors (a multiply and a shift each) behind a uniform
// branch instead of the forty-instruction general division -- on the device this runs ahead of a kernel's first request
__host__ __device__ inline int div_by_splits(int x, int d)
{
    switch (d) {
    case 1: return x;
    case 2: return x >> 1;
    case 3: return x / 3;
    case 4: return x >> 2;
    case 5: return x / 5;
    case 6: return x / 6;
    case 7: return x / 7;
    case 8: return x >> 3;
    default: return x / d;
    }
}
__host__ __device__ inline int attn_fold_chunk(int L, int max_splits)
{
    int sp = (L + 63) >> 6;
    sp = sp > max_splits ? max_splits : sp;
    sp = sp < 1 ? 1 : sp;
    return (div_by_splits(L + sp - 1, sp) + 31) >> 5 << 5;       // L >= 1
}
// splits of `chunk` tokens that hold at least one of the pos + 1 tokens (at most max_splits: no division either)
__host__ __device__ inline int attn_fold_used(int pos, int chunk)
{
    int used = 1;
    while (used * chunk <= pos) ++used;
    return used;
}
enum Epilogue { EPI_F16 = 0, EPI_ROPE_KV = 1, EPI_RESID_F32 = 2, EPI_RESID_F16 = 3, EPI_SWIGLU = 4 };

struct GemvArgs {
    // input rows
    const void *x;                   // [n,k] fp16 (X_F16, X_F16_NORM) or fp32 (X_F32_NORM); unused by X_ATTN_MERGE
    // X_ATTN_MERGE (one row): x = merge of the attention partials [h][part_splits][part_stride floats]: d normalised outputs
    // as fp16, then (max, sum) as fp32 at float index d / 2
    const float *part;
    int32_t part_splits, part_stride, part_chunk;
    int32_t part_used;               // filled in by launch_gemv_reg: splits that hold tokens when the host knows the position
    int32_t units_div, units_mod;    // filled in by launch_gemv_reg: units of a row / wavefronts of the grid, and the remainder
    const uint16_t *norm_w;          // [k] fp16, norm modes only
    float eps;
    // matrix
    union {                          // (the size and the offsets of this block are part of the tuning: one more pointer ahead of
        const uint32_t *q;           // the matrix fields cost the one-row layer 0.3 us per step)
        const uint16_t *wh;          // plain fp16 matrix [m,k] instead of (q, s): launch_gemv_f16w only
    };
    const uint16_t *s;
    int32_t m, k, n;
    int32_t gshift;                  // sub-group (32 columns) index >> gshift = scale index of the row (0: group 32, 1: 64, 2: 128)
    // epilogue
    uint16_t *out_f16;               // EPI_F16: [n,m]; EPI_ROPE_KV: q buffer [n,h*d]; EPI_RESID_F16: out [n,m]; EPI_SWIGLU: act [n,F]
    float *out_f32;                  // EPI_RESID_F32: x1 [n,m]
    const void *resid;               // EPI_RESID_F32: x fp16 [n,m]; EPI_RESID_F16: x1 fp32 [n,m]
    // EPI_ROPE_KV
    uint16_t *kcache, *vcache;
    const float *rope;
    int32_t h, g, d, kv_capacity;
    SeqTable seqs;
    int32_t pos0, slot0;             // position and cache slot of row 0, resolved on the host (what a one-row call needs of seqs)
};

// ---- native 3-bit word layout (gemv_q3.hip describes it): the decode of one group, shared by the kernels that stream it ----
__device__ __forceinline__ uint32_t and_or3(uint32_t w, uint32_t mask, uint32_t bits)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(bits));
    return r;
}
// class of pair p (0: plain, 1: times 8, 2: times 64); pair 15 (columns 30, 31) is plain
__host__ __device__ constexpr int q3n_class(int p) { return p == 15 ? 0 : (p % 5 == 2 ? 2 : (p % 5) % 3 == 1 ? 1 : 0); }

// the 16 fp16 pairs of a group in pair order, each (1024 + f u_even, 1024 + f u_odd) with f = 1, 8 or 64 by class
__device__ __forceinline__ void q3n_decode(uint32_t w0, uint32_t w1, uint32_t w2, uint32_t *pk)
{
    const uint32_t base = 0x64006400u;
    const uint32_t w[3] = {w0, w1, w2};
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t v = w[i], v9 = v >> 9;
        pk[5 * i + 0] = and_or3(v, 0x00070007u, base);
        pk[5 * i + 1] = and_or3(v, 0x00380038u, base);
        pk[5 * i + 2] = and_or3(v, 0x01C001C0u, base);
        pk[5 * i + 3] = and_or3(v9, 0x00070007u, base);
        pk[5 * i + 4] = and_or3(v9, 0x00380038u, base);
    }
    uint32_t t = and_or3(w0 >> 15, 0x00010001u, base);
    t = and_or3(w1 >> 14, 0x00020002u, t);
    pk[15] = and_or3(w2 >> 13, 0x00040004u, t);
}


// weight stream of the register-resident matvec kernel (gemv_reg_kernel.h)
enum { W_Q4 = 0, W_F16 = 1, W_Q3 = 2 };

hipError_t launch_gemv(const GemvArgs &a, int xmode, int epi, hipStream_t stream);
// x-in-registers variant for rows of up to 6 x 2048 columns (gemv_reg_kernel.h, launchers in gemv_q4_reg.hip); launch_gemv picks it when eligible
bool gemv_reg_eligible(const GemvArgs &a);
bool gemv_merge_eligible(const GemvArgs &a);
hipError_t launch_gemv_reg(const GemvArgs &a, int xmode, int epi, hipStream_t stream);
// rows of 12289 .. 32768 columns split over the four wavefronts of a workgroup (gemv_q4_long.hip): plain prologue, row-pair epilogues
bool gemv_long_eligible(const GemvArgs &a, int xmode, int epi);
hipError_t launch_gemv_long(const GemvArgs &a, int epi, hipStream_t stream);
// the same kernel on a plain fp16 matrix (a.wh), one row of x: the fused matvecs of the decode layer of an fp16 model
bool gemv_f16w_eligible(const GemvArgs &a);
bool gemv_f16w_merge_eligible(const GemvArgs &a);
hipError_t launch_gemv_f16w(const GemvArgs &a, int xmode, int epi, hipStream_t stream);
// ... and on 3-bit weights in the native word layout (a.q, a.s with group 32)
bool gemv_q3w_eligible(const GemvArgs &a);
hipError_t launch_gemv_q3w(const GemvArgs &a, int xmode, int epi, hipStream_t stream);

// Workgroup size of the row-norm kernels (one workgroup per row, eight elements per thread and pass) and the order in which the
// per-wavefront sums of squares are added: shared by the stand-alone kernels and the finishing pass that folds the norm in.
// (few rows: a row per workgroup leaves most CUs idle, so the workgroup is as wide as the row allows; many rows: 256 threads)
inline int norm_block_threads(int H, int n) { return n > 128 ? 256 : H >= 8192 ? 1024 : H >= 4096 ? 512 : 256; }
__device__ inline float block_total(const float *red, int waves)
{
    float t = 0.0f;
    for (int w = 0; w < waves; ++w) t += red[w];
    return t;
}
hipError_t launch_rmsnorm(const uint16_t *x, const uint16_t *w, uint16_t *y, int n, int H, float eps, hipStream_t stream);
hipError_t launch_rmsnorm_f32(const float *x, const uint16_t *w, uint16_t *y, int n, int H, float eps, hipStream_t stream);
// element-wise steps as launches of their own (the layer on 3-bit weights): counts are multiples of 8, pointers 16-byte aligned
hipError_t launch_add_rows(const uint16_t *x, const uint16_t *o, float *x1, size_t count, hipStream_t stream);      // x1 = x + o (fp32)
hipError_t launch_add_out(const float *x1, const uint16_t *d, uint16_t *out, size_t count, hipStream_t stream);     // out = fp16(x1 + d)
hipError_t launch_swiglu_rows(const uint16_t *gu, uint16_t *act, int n, int F, hipStream_t stream);                 // act = silu(gate) * up

// MFMA GEMM for large n (gemm_q4_mfma.hip)
constexpr int kGemmMinN = 16;        // rows from which the MFMA GEMM replaces one matvec pass per row
bool gemm_mfma_eligible(const relax_qmat &w, const void *x, int epi);
void gemm_set_waves_per_simd(int v);     // test switch: 2 (default) = eight wavefronts per 256 x 256 tile, 1 = four
constexpr int kSplitKMax = 8;         // k splits of the tiled GEMM at most, when its tiles alone leave more than half of the CUs idle
constexpr int kSplitKMaxN = 512;      // ... and only up to this many rows (the partial tiles are splits * n * m floats)
size_t gemm_splitk_partial_floats(int m, int k, int n, int epi);
// partial: optional workspace of partial_floats fp32 for the k-split form (without it the launch makes one pass over k)
// the same tiled kernel on plain fp16 weights [m,k] (no decode)
bool gemm_f16_eligible(const void *x, const void *w, const void *out, int m, int k);
hipError_t launch_gemm_f16(const uint16_t *x, const uint16_t *w, int n, int m, int k, uint16_t *out, hipStream_t stream);
struct SkinnyFuse;
int gemm_mfma_splits(const relax_qmat &w, int n, int epi, const float *partial, size_t partial_floats);
// fuse: only for a launch that splits (gemm_mfma_splits > 1): the light step folded into its finishing pass
hipError_t launch_gemm_mfma(const uint16_t *x, const relax_qmat &w, int n, int epi, uint16_t *out_f16, float *out_f32, const void *resid,
                            hipStream_t stream, float *partial = nullptr, size_t partial_floats = 0, const SkinnyFuse *fuse = nullptr);
// MFMA matmul for a few rows, split-K with partial tiles in the workspace (gemm_q4_skinny.hip)
constexpr int kSkinnyMinN = 2;       // rows from which the layer takes the matrix path (norm, matmuls, rope as separate launches)
constexpr int kSkinnyMaxN = 128;     // rows up to which the few-row kernel replaces the tiled GEMM
bool gemm_skinny_eligible(const relax_qmat &w, const void *x, int n, int epi);
// Which of the two MFMA kernels takes n rows (Sec. 5.1: the dispatch follows the runtime value of the symbolic dim).  The
// few-row kernel streams the weights once and is the faster one up to 128 rows on matrices of up to ~12k rows; on taller
// matrices the tiled GEMM fills the CUs with tiles of its own and wins earlier (measured, 16-row steps: 22016 x 4096 from 80
// rows, 47 against 63 us; 57344 x 8192 from 48 rows, 146 against 158 us; 12288 x 4096 and smaller: never up to 128 rows).
inline bool gemm_prefers_tiled(int m, int n) { return (n > 64 && m >= 16384) || (n >= 48 && m >= 49152); }
size_t gemm_skinny_partial_floats(int m, int k, int n);
// Optional light step folded into the finishing pass of the few-row matmul (one launch less):
//   residual epilogues: also xn = RMSNorm(result) * norm_w (what the next matmul of the layer, or of the next layer, reads);
//   EPI_F16 on a QKV matrix: rotary embedding of q and k, k and v appended to the cache (q alone is written to out_f16).
struct SkinnyFuse {
    const uint16_t *norm_w;
    uint16_t *xn;
    float eps;
    const relax_layer_dims *dm;
    const relax_kv_cache *cache;
    const SeqTable *st;
};
bool gemm_skinny_fuse_ok(const relax_qmat &w, int epi, const SkinnyFuse &f);
hipError_t launch_skinny_finish(const float *partial, int splits, int n, int m, int epi, uint16_t *out_f16, float *out_f32, const void *resid,
                                hipStream_t stream, const SkinnyFuse *fuse);
hipError_t launch_gemm_skinny(const uint16_t *x, const relax_qmat &w, int n, int epi, uint16_t *out_f16, float *out_f32, const void *resid,
                              float *partial, hipStream_t stream, const SkinnyFuse *fuse = nullptr);
hipError_t launch_rope_append(uint16_t *qkv, const relax_layer_dims &dm, const relax_kv_cache &cache,
                              const SeqTable &st, hipStream_t stream);
hipError_t launch_rope_table(const relax_layer_dims &dm, float *table, hipStream_t stream);
hipError_t launch_unpack(const relax_qmat &w, int8_t *out, hipStream_t stream);
// 3-bit weights: matrix-vector kernel (k a multiple of 32, at most 12288) and the dense decode export
bool gemv_q3_supported(int m, int k);
hipError_t launch_gemv_q3(const uint16_t *x, const relax_qmat &w, int n, uint16_t *out, hipStream_t stream);
hipError_t launch_unpack_q3(const relax_qmat &w, int8_t *out, hipStream_t stream);
// native 3-bit layout (gemv_q3.hip): one-time repack, its dense decode export, the streaming matvec for 1..n rows of x
hipError_t launch_repack_q3(const relax_qmat &canonical, uint32_t *dst, hipStream_t stream);
hipError_t launch_unpack_q3_native(const relax_qmat &w, int8_t *out, hipStream_t stream);
hipError_t launch_gemv_q3_native(const uint16_t *x, const relax_qmat &w, int n, uint16_t *out, hipStream_t stream);
// the tiled MFMA GEMM on native 3-bit weights (gemm_q4_mfma.hip), taken from kQ3GemmRows rows of x on
constexpr int kQ3GemmRows = 16;
bool gemm_q3_eligible(const void *x, const relax_qmat &w, const void *out);
hipError_t launch_gemm_q3(const uint16_t *x, const relax_qmat &w, int n, uint16_t *out, hipStream_t stream);
hipError_t launch_dequantize(const relax_qmat &w, float *out, hipStream_t stream);

// Split-L attention: chunk length and split count are pure functions of the runtime shape.
struct AttnPlan {
    int32_t chunk;                   // tokens per split
    int32_t splits;                  // grid extent along L (rows with fewer tokens leave the tail idle)
};
AttnPlan attn_plan(int32_t n, int32_t g, int32_t L_max);
size_t attn_partial_floats(const relax_layer_dims &dm, int32_t n_max, int32_t L_max);
bool attn_mha_split_supported(const relax_layer_dims &dm);
hipError_t launch_attention_mha_split(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm,
                                      const SeqTable &st, int32_t chunk, int32_t splits, int32_t part_stride, float *partials, hipStream_t stream);
hipError_t launch_attention(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm,
                            const SeqTable &st, int32_t L_max, uint16_t *out, float *partials, hipStream_t stream);

// MFMA split kernel for grouped-query decode rows (attn_gqa.hip); partials in the format of the scalar split kernel
bool attn_gqa_supported(const relax_layer_dims &dm);
hipError_t launch_attention_gqa_split(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm,
                                      const SeqTable &st, const AttnPlan &pl, float *partials, hipStream_t stream);

// Causal MFMA attention for calls with many rows per sequence (attn_prefill.hip)
constexpr int kPrefillMinQ = 16;     // longest q_len from which launch_attention takes the MFMA kernel
bool attn_prefill_supported(const relax_layer_dims &dm);
hipError_t launch_attention_prefill(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm,
                                    const SeqTable &st, uint16_t *out, hipStream_t stream);

// Model wrapper steps (model_head.hip)
hipError_t launch_embed(const int32_t *ids, const uint16_t *E, uint16_t *x, int n, int H, int V, uint32_t *err, hipStream_t stream);
hipError_t launch_final_norm(const uint16_t *x, const uint16_t *w, uint16_t *y, const SeqTable &st, int H, float eps, hipStream_t stream);
int lm_head_rows_per_pass(int H);    // rows of x one pass of the fp16 matvec kernel holds in LDS (at most 8)
hipError_t launch_lm_head(const uint16_t *xn, const uint16_t *W, uint16_t *logits, int B, int H, int V, int n_cus, hipStream_t stream);
hipError_t launch_argmax(const uint16_t *logits, int32_t *ids, int B, int V, hipStream_t stream);

// Device-ceiling probes (probes.hip)
hipError_t launch_probe_stream_read(const void *buf, size_t bytes, uint32_t *sink, int n_cus, hipStream_t stream);
hipError_t launch_probe_mfma(float *sink, int iters, int random_data, int n_cus, hipStream_t stream);

// ---- front of every layer / model workspace --------------------------------------------------------------------
// One 256-byte line of flags the kernels may raise (word 0 bit 1: a token id outside the vocabulary was read as id 0);
// relax_workspace_init clears it, relax_workspace_error reads it.
constexpr size_t kWsFlagBytes = 256;
hipError_t launch_ws_clear(void *base, size_t bytes, hipStream_t stream);
// Writes a chunk of the ragged descriptor into the device table [4][B] (batches that do not ride in kernel arguments).
constexpr int kTableChunk = 32;
struct TableChunk {
    int32_t first, count, B;
    int32_t q_start[kTableChunk], q_len[kTableChunk], kv_len[kTableChunk], slot[kTableChunk];
};
hipError_t launch_table_write(int32_t *table, const TableChunk &chunk, hipStream_t stream);

// A quantised matrix as the streaming kernels pass it around
struct DLMat {
    const uint32_t *q;
    const uint16_t *s;
    int32_t m, k;
    int32_t gshift;
};

}  // namespace relax
