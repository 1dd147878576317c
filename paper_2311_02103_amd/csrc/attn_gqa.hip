// Split-L decode attention for grouped-query layouts (several query heads per KV head): the query heads of a KV
// head form the columns of an MFMA tile, so every K/V byte is loaded once and meets all of them on the matrix cores
// instead of in per-head scalar loops (Relax, Sec. 4.2 fused attention operator with a symbolic KV length; Sec. 5.1
// batched decode).  Same split plan and partial format as the scalar split kernel, same merge kernel.
//
// A workgroup is one (row, KV head, split along L); each of its four wavefronts walks its own 32-token tiles with no
// workgroup barrier in the loop:
//   S^T[t, head] = K[t, :] . Q[head, :]   A operand = the K tile straight from global memory (lane = token t % 32;
//                                          k step ks takes d = 16 ks + 8 (l / 32) .. + 8), B operand = the query
//                                          heads in the same order, read from LDS (written once per workgroup);
//   online softmax per column (= per head) inside a lane plus one exchange with lane ^ 32;
//   O^T[d, head] += V^T[d, t] . P^T[t, head]   A operand = the V tile, staged in a wavefront-private LDS region and
//                                          read with the LDS transpose read of gfx950 (lane r of a 16-lane block
//                                          addresses V[t0 + r/4][d0 + 4 (r%4)], lane L receives V[t0..t0+3][d0 + L]);
//                                          B operand = the probabilities the lane already holds.
// Columns beyond the number of heads per group re-read the last head and are dropped.
#include "relax_common.h"

namespace relax {

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kGqaMaxRep = 16;       // query heads per KV head this kernel serves (the merge of the four wavefronts reuses the V region)

// grid: x = KV head, y = split along L, z = row of the call
template <int D>
__global__ __launch_bounds__(256, 2) void attn_gqa_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ kc,
                                                       const uint16_t *__restrict__ vc, float *__restrict__ part, SeqTable st,
                                                       int h, int g, int cap, int chunk, int splits, int q_stride)
{
    constexpr int KS = D / 16;       // k steps of K Q^T
    constexpr int DB = D / 32;       // 32-wide blocks of the head dimension in O^T
    constexpr int VP = D + 32;       // V tile pitch in halfs (distinct banks for the transpose reads of a 32-lane half)
    constexpr int VPK = 32 * (D / 8) / 64;          // 16-byte V packets per lane and tile
    __shared__ __align__(16) uint16_t vs_all[4 * 32 * VP];

    const int i = blockIdx.z, split = blockIdx.y, kvh = blockIdx.x;
    const RowInfo ri = row_info(st, i);
    const int L = ri.pos + 1;
    const int t_begin = split * chunk;
    if (t_begin >= L) return;                                  // uniform for the workgroup
    const int t_end = min(L, t_begin + chunk);
    const int rep = h / g;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hf = lane >> 5;
    const float scale = 1.0f / sqrtf((float)D);

    uint16_t *vs = vs_all + wave * 32 * VP;
    const size_t slot_base = (size_t)ri.slot * cap;
    const int tr_row = hf * 4 + ((lane & 15) >> 2), tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;

    // registers of one tile in flight: the lane's run of its K row (KS packets) and its share of the V tile
    u32x4_t kreg[KS], vreg[VPK];
    auto tile_load = [&](int t0) {                             // rows are clamped to the split: masked later
        const size_t krow = ((slot_base + min(t0 + col, t_end - 1)) * g + kvh) * D + hf * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[ks] = *(const u32x4_t *)(kc + krow + ks * 16);
#pragma unroll
        for (int p = 0; p < VPK; ++p) {
            const int pk = lane + p * 64, r = pk / (D / 8), c = pk % (D / 8);
            vreg[p] = stream_load((const u32x4_t *)(vc + ((slot_base + min(t0 + r, t_end - 1)) * g + kvh) * D + c * 8));
        }
    };

    // the first K / V tile is requested before the Q fragments are staged: it does not depend on them, and a workgroup
    // lives for a few tiles only
    const int t_first = t_begin + wave * 32;
    if (t_first < t_end) tile_load(t_first);
    // ---- Q fragments: lane owns head (col) of the group; k step ks pairs d = 16 ks + 8 hf .. + 8 of K and Q.
    // The same for every wavefront and every tile: kept in LDS (KS x 64 lanes x 16 bytes), not in registers, so that
    // two workgroups fit a CU ----
    __shared__ __align__(16) uint16_t q_lds[KS * 64 * 8];
    if (wave == 0) {
        const int head = kvh * rep + min(col, rep - 1);
        const uint16_t *src = q + (size_t)i * q_stride + (size_t)head * D + hf * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) *(half8_t *)(q_lds + (ks * 64 + lane) * 8) = *(const half8_t *)(src + ks * 16);
    }
    __syncthreads();

    float16_t O[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) O[db][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    for (int t0 = t_first; t0 < t_end; t0 += 128) {
        // ---- S^T = K Q^T on the tile in registers; V tile to the wavefront's LDS region ----
        float16_t S;
#pragma unroll
        for (int v = 0; v < 16; ++v) S[v] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) S = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, kreg[ks]), *(const half8_t *)(q_lds + (ks * 64 + lane) * 8), S, 0, 0, 0);
#pragma unroll
        for (int p = 0; p < VPK; ++p) {
            const int pk = lane + p * 64, r = pk / (D / 8), c = pk % (D / 8);
            *(u32x4_t *)(vs + r * VP + c * 8) = vreg[p];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");      // the wavefront's own LDS traffic is in order
        if (t0 + 128 < t_end) tile_load(t0 + 128);
        // ---- mask, online softmax per column; P^T packed as the B operand of the second product ----
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int t = t0 + 8 * (v >> 2) + 4 * hf + (v & 3);
            const float s = t < t_end ? S[v] * scale : -INFINITY;
            S[v] = s;
            mx = fmaxf(mx, s);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
        constexpr float kSlack = 6.0f;                         // lazy rescaling: see the prefill kernel
        const bool move = mx > m_run + kSlack;
        const float m_new = move ? mx : m_run;
        const float alpha = move ? __expf(m_run - m_new) : 1.0f;
        half8_t pf[2];
        float psum = 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float p = __expf(S[v] - m_new);
            psum += p;
            pf[v >> 3][v & 7] = (_Float16)p;
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__any(move)) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) O[db][v] *= alpha;
        }
        // ---- O^T += V^T P^T ----
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const uint16_t *vp = vs + (s2 * 16 + tr_row) * VP + db * 32 + tr_col;
                const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t *)vp);
                const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t *)(vp + 8 * VP));
                const half8_t vf = __builtin_bit_cast(half8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                O[db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[s2], O[db], 0, 0, 0);
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");      // reads done before the next tile overwrites the region
    }

    // ---- merge the four wavefronts through LDS (the V regions are free now) and write the partial of (row, head, split) ----
    __syncthreads();
    float *sm = reinterpret_cast<float *>(vs_all);             // [4][rep][D + 2]
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    if (col < rep) {
        float *dst = sm + (wave * rep + col) * (D + 2);
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[db * 32 + 8 * (v >> 2) + 4 * hf + (v & 3)] = O[db][v];
        if (hf == 0) dst[D] = m_run, dst[D + 1] = l_tot;
    }
    __syncthreads();
    for (int idx = tid; idx < rep * D; idx += 256) {
        const int r = idx / D, e = idx - r * D;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mm = fmaxf(mm, sm[(w * rep + r) * (D + 2) + D]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float *src = sm + (w * rep + r) * (D + 2);
            const float sc = (src[D] == -INFINITY) ? 0.0f : __expf(src[D] - mm);
            num += src[e] * sc;
            den += src[D + 1] * sc;
        }
        float *dst = part + (((size_t)i * h + kvh * rep + r) * splits + split) * (D + 2);
        dst[e] = num;
        if (e == 0) dst[D] = mm, dst[D + 1] = den;
    }
}

}  // namespace

bool attn_gqa_supported(const relax_layer_dims &dm)
{
    const int rep = dm.n_heads / dm.n_kv_heads;
    return rep >= 4 && rep <= kGqaMaxRep && (dm.head_dim == 128 || dm.head_dim == 64);
}

hipError_t launch_attention_gqa_split(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm,
                                      const SeqTable &st, const AttnPlan &pl, float *partials, hipStream_t stream)
{
    dim3 grid(dm.n_kv_heads, pl.splits, st.n);
    if (dm.head_dim == 128)
        hipLaunchKernelGGL(attn_gqa_kernel<128>, grid, dim3(256), 0, stream, q, cache.k, cache.v, partials, st, dm.n_heads, dm.n_kv_heads,
                           dm.kv_capacity, pl.chunk, pl.splits, q_stride);
    else
        hipLaunchKernelGGL(attn_gqa_kernel<64>, grid, dim3(256), 0, stream, q, cache.k, cache.v, partials, st, dm.n_heads, dm.n_kv_heads,
                           dm.kv_capacity, pl.chunk, pl.splits, q_stride);
    return hipGetLastError();
}

}  // namespace relax
