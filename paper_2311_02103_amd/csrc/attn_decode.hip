// Attention over a KV cache of symbolic length, split along L ("flash-decoding" shape):
// the paper treats attention as one fused operator whose KV length is a runtime value
// (Relax, Sec. 4.2 custom attention pattern; Sec. 5.1 dynamic sequence length).  A decode row
// reads L * g * d * 2 * 2 bytes of cache and does almost no arithmetic, so the kernel is a
// streaming read: L is cut into chunks across workgroups so that 256 CUs have work even at
// batch 1, every K/V byte is loaded once with 16-byte loads (all query heads of a KV head are
// served by the same load), and each workgroup leaves an un-normalised partial (running max,
// running sum, accumulator) in the caller's workspace (Sec. 4.4: kernel scratch lifted to the
// caller).  A second small kernel merges the partials of a (row, head) with the usual
// max-rescaling.  Scores, softmax and accumulation are fp32.
#include "relax_common.h"

namespace relax {

AttnPlan attn_plan(int32_t n, int32_t g, int32_t L_max)
{
    long long total = (long long)n * g * (L_max > 0 ? L_max : 1);
    long long c = (total + 1023) / 1024;
    c = ((c + 63) / 64) * 64;
    if (c < 64) c = 64;
    if (c > 512) c = 512;
    AttnPlan p;
    p.chunk = (int32_t)c;
    p.splits = (L_max + p.chunk - 1) / p.chunk;
    if (p.splits < 1) p.splits = 1;
    return p;
}

// Upper bound over every (n <= n_max, L <= L_max) of n*h*splits*(d+2) floats; see attn_plan:
// unclamped chunks give at most 1024/(n g) + 1 splits, chunks clamped at 512 give ceil(L/512).
size_t attn_partial_floats(const relax_layer_dims &dm, int32_t n_max, int32_t L_max)
{
    const size_t h = dm.n_heads, rep = dm.n_heads / dm.n_kv_heads;
    size_t a = rep * 1024 + (size_t)n_max * h;
    size_t b = (size_t)n_max * h * (size_t)((L_max + 511) / 512);
    return (a > b ? a : b) * (size_t)(dm.head_dim + 2);
}

__device__ inline void unpack8(const uint4 &raw, float *f)
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[2 * j] = h2f((uint16_t)(w[j] & 0xFFFFu));
        f[2 * j + 1] = h2f((uint16_t)(w[j] >> 16));
    }
}

// merge state b into state a (running max m, running sum l, accumulator acc[8])
__device__ inline void merge_state(float &ma, float &la, float *acca, float mb, float lb, const float *accb)
{
    const float mn = fmaxf(ma, mb);
    const float sa = (ma == -INFINITY) ? 0.0f : __expf(ma - mn);
    const float sb = (mb == -INFINITY) ? 0.0f : __expf(mb - mn);
    la = la * sa + lb * sb;
#pragma unroll
    for (int e = 0; e < 8; ++e) acca[e] = acca[e] * sa + accb[e] * sb;
    ma = mn;
}

// grid: x = KV head * (rep/REP) + head sub-group, y = split along L, z = row of the call
template <int D, int REP>
__global__ __launch_bounds__(256) void attn_split_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ kc,
                                                         const uint16_t *__restrict__ vc, float *__restrict__ part, SeqTable st,
                                                         int h, int g, int cap, int chunk, int splits, int q_stride)
{
    constexpr int LPT = D / 8;        // lanes that share one token (each owns 8 of its d elements)
    constexpr int TPW = kWave / LPT;  // tokens per wavefront step
    __shared__ float sm[4 * REP * (D + 2)];

    const int i = blockIdx.z, split = blockIdx.y;
    const RowInfo ri = row_info(st, i);
    const int L = ri.pos + 1;
    const int t_begin = split * chunk;
    if (t_begin >= L) return;                                  // uniform for the workgroup
    const int t_end = min(L, t_begin + chunk);

    const int rep = h / g, subs = rep / REP;
    const int kvh = blockIdx.x / subs, head0 = kvh * rep + (blockIdx.x - kvh * subs) * REP;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int sub = lane / LPT, e0 = (lane % LPT) * 8;
    const float inv_sqrt_d = 1.0f / sqrtf((float)D);

    float qf[REP][8], acc[REP][8], m[REP], l[REP];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
        unpack8(*(const uint4 *)(q + (size_t)i * q_stride + (size_t)(head0 + r) * D + e0), qf[r]);
        m[r] = -INFINITY;
        l[r] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.0f;
    }

    const size_t slot_base = (size_t)ri.slot * cap;
    for (int t = t_begin + wave * TPW + sub; t < t_end; t += 4 * TPW) {
        const size_t at = ((slot_base + t) * g + kvh) * D + e0;
        float kf[8], vf[8];
        unpack8(stream_load((const uint4 *)(kc + at)), kf);
        unpack8(stream_load((const uint4 *)(vc + at)), vf);
#pragma unroll
        for (int r = 0; r < REP; ++r) {
            float dot = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) dot += qf[r][e] * kf[e];
#pragma unroll
            for (int off = LPT / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, kWave);
            const float s = dot * inv_sqrt_d;
            const float mn = fmaxf(m[r], s);
            const float ca = __expf(m[r] - mn);                // m = -inf on the first token: exp(-inf) = 0
            const float p = __expf(s - mn);
            l[r] = l[r] * ca + p;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] = acc[r][e] * ca + p * vf[e];
            m[r] = mn;
        }
    }

    // merge the TPW token groups of the wavefront (lanes that own the same 8 elements)
#pragma unroll
    for (int r = 0; r < REP; ++r) {
#pragma unroll
        for (int off = LPT; off < kWave; off <<= 1) {
            float mb = __shfl_xor(m[r], off, kWave), lb = __shfl_xor(l[r], off, kWave), accb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) accb[e] = __shfl_xor(acc[r][e], off, kWave);
            merge_state(m[r], l[r], acc[r], mb, lb, accb);
        }
        if (lane < LPT) {
            float *dst = sm + (wave * REP + r) * (D + 2);
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e0 + e] = acc[r][e];
            if (lane == 0) {
                dst[D] = m[r];
                dst[D + 1] = l[r];
            }
        }
    }
    __syncthreads();

    // merge the four wavefronts and write the partial of (row, head, split)
    for (int idx = tid; idx < REP * D; idx += 256) {
        const int r = idx / D, e = idx - r * D;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mm = fmaxf(mm, sm[(w * REP + r) * (D + 2) + D]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float *src = sm + (w * REP + r) * (D + 2);
            const float sc = (src[D] == -INFINITY) ? 0.0f : __expf(src[D] - mm);
            num += src[e] * sc;
            den += src[D + 1] * sc;
        }
        float *dst = part + (((size_t)i * h + head0 + r) * splits + split) * (D + 2);
        dst[e] = num;
        if (e == 0) {
            dst[D] = mm;
            dst[D + 1] = den;
        }
    }
}

// ---- split kernel for one query head per KV head (multi-head attention) -----------------------------------------------
//
// Same work split and partial format as attn_split_kernel, built for the memory system: a wavefront step is 4 K loads
// and 4 V loads of 16 bytes per lane (TS tokens), two steps are in flight, and the first two are requested before
// anything else, so at the usual chunk sizes (a wavefront owns two to eight steps) most of the chunk is already on its
// way when the first score is computed.  q . k runs on packed fp16 pairs with v_dot2_f32_f16 (exact products, fp32
// sums) and is reduced over the lanes of a token with DPP row operations; the softmax state advances once per step
// (one rescale for TS tokens instead of one per token).  The step schedule is straight-line in its loads (no load
// under a condition that merges back), so a wait counts exactly the loads requested after the step it needs.
typedef uint32_t u32x4a_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2a_t __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

template <int D, bool HALF>
__global__ __launch_bounds__(256) void attn_mha_split_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ kc,
                                                             const uint16_t *__restrict__ vc, float *__restrict__ part, SeqTable st,
                                                             int h, int cap, int chunk, int splits, int q_stride, int ps, int pos0,
                                                             int slot0)
{
    constexpr int LPT = D / 8;        // lanes that share one token (each owns 8 of its d elements)
    constexpr int TPW = kWave / LPT;  // tokens per load instruction of a wavefront
    constexpr int NL = 4;             // K (and V) loads per step
    constexpr int TS = NL * TPW;      // tokens per wavefront step
    __shared__ float sm[4 * (D + 2)];
    // every kernel argument in scalar registers here: one round of scalar loads and one wait ahead of the first K / V
    // request, instead of a round per group of arguments at the place of its first use
    asm volatile("" ::"s"(q), "s"(kc), "s"(vc), "s"(part), "s"(h), "s"(cap), "s"(chunk), "s"(splits), "s"(q_stride), "s"(ps), "s"(pos0),
                 "s"(slot0));

    const int i = blockIdx.z, split = blockIdx.y, head = blockIdx.x;
    RowInfo ri = {0, pos0, slot0};                             // pos0 >= 0: the only row of the call, resolved by the host
    if (pos0 < 0) ri = row_info(st, i);
    const int L = ri.pos + 1;
    if (chunk <= 0) chunk = attn_fold_chunk(L, splits);        // device-resident descriptor: the plan follows the L read here
    const int t_begin = split * chunk;
    if (t_begin >= L) return;                                  // uniform for the workgroup
    const int t_end = min(L, t_begin + chunk);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int sub = lane / LPT, e0 = (lane % LPT) * 8;
    const float inv_sqrt_d = 1.0f / sqrtf((float)D);

    // step s of this wavefront covers tokens t_begin + (4 s + wave) TS .. + TS - 1
    const int first = t_begin + wave * TS;
    const int ns = first < t_end ? (t_end - first + 4 * TS - 1) / (4 * TS) : 0;
    // Addresses: a uniform base per (slot, head) plus a 32-bit byte offset per lane that K and V share (the launcher
    // checks that a slot of the cache stays under 2 GiB).  The offsets of a step are those of the step before plus a
    // constant, clamped to the last token of the split: two vector instructions per K / V pair instead of a 64-bit
    // multiply-add each, ahead of the first request as well as in the stream.
    const uint32_t row_bytes = (uint32_t)h * D * 2;            // one token of the cache, all heads
    const size_t slot_base = ((size_t)ri.slot * cap) * ((size_t)h * D) + (size_t)head * D;
    const char *kslot = (const char *)(kc + slot_base), *vslot = (const char *)(vc + slot_base);
    const uint32_t last_off = (uint32_t)(t_end - 1) * row_bytes + (uint32_t)e0 * 2;
    const uint32_t step_bytes = 4 * TS * row_bytes;
    uint32_t run[NL];                                          // offsets of the next step to request, not clamped
#pragma unroll
    for (int j = 0; j < NL; ++j) run[j] = (uint32_t)(first + sub + j * TPW) * row_bytes + (uint32_t)e0 * 2;

    struct Step {
        u32x4a_t k[NL], v[NL];
    };
    // requests step s; the calls come in the order s = 0, 1, 2, ..
    auto step_load = [&](Step &sp, int) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            const uint32_t at = min(run[j], last_off);         // tokens past the end re-read the last one, masked below
            sp.k[j] = stream_load((const u32x4a_t *)(kslot + at));
            sp.v[j] = stream_load((const u32x4a_t *)(vslot + at));
            run[j] += step_bytes;
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    Step sa, sb;
    step_load(sa, 0);
    step_load(sb, 1);
    const u32x4a_t qv = *(const u32x4a_t *)(q + (size_t)i * q_stride + (size_t)head * D + e0);

    float acc[8], m = -INFINITY, l = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.0f;

    auto consume = [&](const Step &sp, int s) {
        const int t0 = first + s * 4 * TS + sub;
        float sc[NL];
        float mx = m;
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            float dot = 0.0f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t kw = sp.k[j][w], qw = qv[w];    // element copies: a bit_cast applied to the subscript itself reads word 0
                dot = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2a_t, kw), __builtin_bit_cast(half2a_t, qw), dot, false);
            }
            dot += dpp_f<0xB1>(dot);                           // lane ^ 1
            dot += dpp_f<0x4E>(dot);                           // lane ^ 2
            if (LPT == 16) {
                dot += dpp_f<0x124>(dot);                      // rotate the row of 16 by 4, then by 8
                dot += dpp_f<0x128>(dot);
            } else {
                dot += dpp_f<0x141>(dot);                      // mirror within the half row of 8
            }
            sc[j] = (t0 + j * TPW < t_end) ? dot * inv_sqrt_d : -INFINITY;
            mx = fmaxf(mx, sc[j]);
        }
        const float mref = (mx == -INFINITY) ? 0.0f : mx;      // nothing valid yet: every weight below is exp(-inf) = 0
        const float ca = __expf(m - mref);
        float p[NL], psum = 0.0f;
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            p[j] = __expf(sc[j] - mref);
            psum += p[j];
        }
        l = l * ca + psum;
        m = mx;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] *= ca;
#pragma unroll
        for (int j = 0; j < NL; ++j)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t vw = sp.v[j][w];
                const half2a_t vv = __builtin_bit_cast(half2a_t, vw);
                acc[2 * w] += p[j] * (float)vv.x;
                acc[2 * w + 1] += p[j] * (float)vv.y;
            }
    };

    const int nq = ns >> 1;
    int s = 0;
#pragma unroll 1
    for (; s + 2 < 2 * nq; s += 2) {
        consume(sa, s);
        step_load(sa, s + 2);
        consume(sb, s + 1);
        step_load(sb, s + 3);
    }
    if (nq > 0) {
        if (ns & 1) {
            consume(sa, s);
            step_load(sa, s + 2);
            consume(sb, s + 1);
            consume(sa, s + 2);
        } else {
            consume(sa, s);
            consume(sb, s + 1);
        }
    } else if (ns == 1) {
        consume(sa, 0);
    }

    // merge the TPW token groups of the wavefront (lanes that own the same 8 elements)
#pragma unroll
    for (int off = LPT; off < kWave; off <<= 1) {
        float mb = __shfl_xor(m, off, kWave), lb = __shfl_xor(l, off, kWave), accb[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) accb[e] = __shfl_xor(acc[e], off, kWave);
        merge_state(m, l, acc, mb, lb, accb);
    }
    if (lane < LPT) {
        float *dst = sm + wave * (D + 2);
#pragma unroll
        for (int e = 0; e < 8; ++e) dst[e0 + e] = acc[e];
        if (lane == 0) dst[D] = m, dst[D + 1] = l;
    }
    __syncthreads();
    // merge the four wavefronts and write the partial of (row, head, split)
    if (tid < D) {
        const int e = tid;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) mm = fmaxf(mm, sm[w * (D + 2) + D]);
        float num = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float *src = sm + w * (D + 2);
            const float scw = (src[D] == -INFINITY) ? 0.0f : __expf(src[D] - mm);
            num += src[e] * scw;
            den += src[D + 1] * scw;
        }
        float *dst = part + (((size_t)i * h + head) * splits + split) * ps;          // ps floats per partial
        if (HALF) {
            // for a reader that folds the merge into its prologue: out_s = acc_s / l_s as fp16 (D halfs), then (m_s, l_s)
            reinterpret_cast<uint16_t *>(dst)[e] = f2h(num / den);                       // den > 0: the split holds at least one token
            if (e == 0) dst[D / 2] = mm, dst[D / 2 + 1] = den;
        } else {
            dst[e] = num;                                                                // ps >= D + 2
            if (e == 0) dst[D] = mm, dst[D + 1] = den;
        }
    }
}

// one workgroup of D threads per (row, head): out = sum_s acc_s e^(m_s - M) / sum_s l_s e^(m_s - M).
// No LDS and no barrier: a thread reads the (m, l) pair of every split itself (the same address for the whole
// workgroup: one transaction) next to its own accumulator element, 16 splits per round with all loads of a round in
// flight together, and folds a round in with the usual max-rescaling.
template <int D>
__global__ void attn_merge_kernel(const float *__restrict__ part, uint16_t *__restrict__ out, SeqTable st, int h, int chunk,
                                  int splits)
{
    constexpr int RS = 16;
    const int i = blockIdx.x / h, e = threadIdx.x;
    const RowInfo ri = row_info(st, i);
    const int used = (ri.pos + chunk) / chunk;                 // ceil((pos+1)/chunk)
    const float *src = part + (size_t)blockIdx.x * splits * (D + 2);
    float mm = -INFINITY, num = 0.0f, den = 0.0f;
    for (int s0 = 0; s0 < used; s0 += RS) {
        float ms[RS], ls[RS], as[RS];
#pragma unroll
        for (int j = 0; j < RS; ++j) {
            const float *p = src + (size_t)min(s0 + j, used - 1) * (D + 2);
            ms[j] = p[D], ls[j] = p[D + 1], as[j] = p[e];
        }
        float mx = mm;
#pragma unroll
        for (int j = 0; j < RS; ++j) mx = (s0 + j < used) ? fmaxf(mx, ms[j]) : mx;
        const float mref = (mx == -INFINITY) ? 0.0f : mx;
        const float c0 = __expf(mm - mref);
        num *= c0, den *= c0;
#pragma unroll
        for (int j = 0; j < RS; ++j) {
            const float w = (s0 + j < used) ? __expf(ms[j] - mref) : 0.0f;
            num += as[j] * w, den += ls[j] * w;
        }
        mm = mx;
    }
    out[(size_t)blockIdx.x * D + e] = f2h(num / den);
}

template <int D, int REP>
static hipError_t launch_split(const uint16_t *q, int q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm, const SeqTable &st,
                               const AttnPlan &pl, float *partials, hipStream_t stream)
{
    const int rep = dm.n_heads / dm.n_kv_heads;
    dim3 grid(dm.n_kv_heads * (rep / REP), pl.splits, st.n);
    hipLaunchKernelGGL((attn_split_kernel<D, REP>), grid, dim3(256), 0, stream, q, cache.k, cache.v, partials, st, dm.n_heads,
                       dm.n_kv_heads, dm.kv_capacity, pl.chunk, pl.splits, q_stride);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_d(const uint16_t *q, int q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm, const SeqTable &st,
                           const AttnPlan &pl, uint16_t *out, float *partials, hipStream_t stream)
{
    const int rep = dm.n_heads / dm.n_kv_heads;
    hipError_t e;
    if (attn_gqa_supported(dm)) e = launch_attention_gqa_split(q, q_stride, cache, dm, st, pl, partials, stream);   // MFMA kernel for grouped heads
    else if (rep == 1 && attn_mha_split_supported(dm)) {
        const HostRow hr = host_row(st);
        hipLaunchKernelGGL((attn_mha_split_kernel<D, false>), dim3(dm.n_heads, pl.splits, st.n), dim3(256), 0, stream, q, cache.k, cache.v, partials, st,
                           dm.n_heads, dm.kv_capacity, pl.chunk, pl.splits, q_stride, D + 2, hr.pos, hr.slot);
        e = hipGetLastError();
    }
    else if (rep % 8 == 0) e = launch_split<D, 8>(q, q_stride, cache, dm, st, pl, partials, stream);
    else if (rep % 4 == 0) e = launch_split<D, 4>(q, q_stride, cache, dm, st, pl, partials, stream);
    else if (rep % 2 == 0) e = launch_split<D, 2>(q, q_stride, cache, dm, st, pl, partials, stream);
    else e = launch_split<D, 1>(q, q_stride, cache, dm, st, pl, partials, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((attn_merge_kernel<D>), dim3(st.n * dm.n_heads), dim3(D), 0, stream, partials, out, st, dm.n_heads,
                       pl.chunk, pl.splits);
    return hipGetLastError();
}

// split kernel alone, for a caller that folds the merge into its own prologue (one query head per KV head, decode rows):
// partial of (row, head, split) at partials + ((row * h + head) * splits + split) * part_stride floats, in the half
// format: head_dim normalised outputs acc / l as fp16, then (max, sum) as fp32 at float index head_dim / 2; part_stride >= head_dim / 2 + 2
bool attn_mha_split_supported(const relax_layer_dims &dm)
{
    // 32-bit byte offsets inside a slot of the cache (plus the two steps a wavefront requests past its split)
    const size_t slot_bytes = ((size_t)dm.kv_capacity + 256) * dm.n_kv_heads * dm.head_dim * 2;
    return dm.n_heads == dm.n_kv_heads && (dm.head_dim == 128 || dm.head_dim == 64) && slot_bytes < ((size_t)1 << 31);
}

hipError_t launch_attention_mha_split(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm,
                                      const SeqTable &st, int32_t chunk, int32_t splits, int32_t part_stride, float *partials, hipStream_t stream)
{
    const dim3 grid(dm.n_heads, splits, st.n);
    const HostRow hr = host_row(st);
    if (dm.head_dim == 128)
        hipLaunchKernelGGL((attn_mha_split_kernel<128, true>), grid, dim3(256), 0, stream, q, cache.k, cache.v, partials, st, dm.n_heads,
                           dm.kv_capacity, chunk, splits, q_stride, part_stride, hr.pos, hr.slot);
    else
        hipLaunchKernelGGL((attn_mha_split_kernel<64, true>), grid, dim3(256), 0, stream, q, cache.k, cache.v, partials, st, dm.n_heads,
                           dm.kv_capacity, chunk, splits, q_stride, part_stride, hr.pos, hr.slot);
    return hipGetLastError();
}

hipError_t launch_attention(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm, const SeqTable &st,
                            int32_t L_max, uint16_t *out, float *partials, hipStream_t stream)
{
    if (st.q_max >= kPrefillMinQ && attn_prefill_supported(dm)) return launch_attention_prefill(q, q_stride, cache, dm, st, out, stream);
    const AttnPlan pl = attn_plan(st.n, dm.n_kv_heads, L_max);
    if (dm.head_dim == 128) return launch_d<128>(q, q_stride, cache, dm, st, pl, out, partials, stream);
    if (dm.head_dim == 64) return launch_d<64>(q, q_stride, cache, dm, st, pl, out, partials, stream);
    return hipErrorInvalidValue;
}

}  // namespace relax
