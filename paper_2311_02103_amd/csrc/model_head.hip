// The steps of a model step outside the decoder layers (embedding gather, final RMSNorm on the last row of each
// sequence, fp16 LM head, greedy pick).  At decode the LM head is one more HBM stream per token (vocab x hidden
// fp16, 262 MB for the 7B shape): the same batch-1 matrix-vector special case the paper singles out (Relax,
// Sec. 5.1), here with unquantised weights.
#include <atomic>

#include "relax_common.h"

namespace relax {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ inline float dot2h(uint32_t a_bits, uint32_t b_bits, float acc)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a_bits), __builtin_bit_cast(half2_t, b_bits), acc, false);
}

// x[i,:] = E[ids[i],:].  An id outside [0, V) raises the workspace error flag and reads row 0 instead.
__global__ __launch_bounds__(256) void embed_kernel(const int32_t *__restrict__ ids, const uint16_t *__restrict__ E,
                                                    uint16_t *__restrict__ x, int H, int V, uint32_t *err)
{
    int id = ids[blockIdx.x];
    if (id < 0 || id >= V) {
        if (threadIdx.x == 0) atomicOr(err, 2u);
        id = 0;
    }
    const u32x4_t *src = (const u32x4_t *)(E + (size_t)id * H);
    u32x4_t *dst = (u32x4_t *)(x + (size_t)blockIdx.x * H);
    for (int c = threadIdx.x; c < H / 8; c += 256) dst[c] = src[c];
}

// y[b,:] = RMSNorm(x[last row of sequence b,:]) * w; one workgroup per sequence, fp32 reduction.
__global__ __launch_bounds__(256) void final_norm_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ w,
                                                         uint16_t *__restrict__ y, SeqTable st, int H, float eps)
{
    __shared__ float red[4];
    const int b = blockIdx.x;
    int row;
    if (st.dev) {
        row = st.dev[b] + st.dev[st.B + b] - 1;
    } else {
        row = 0;
#pragma unroll
        for (int j = 0; j < kInlineSeqs; ++j)
            if (j == b) row = st.q_start[j] + st.q_len[j] - 1;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t base = (size_t)row * H;
    // rows of whole 16-byte packets, at most kNormPasses per thread: the row stays in registers between the two passes
    constexpr int kNormPasses = 4;
    const bool vec = (H % 8 == 0) && H <= 256 * 8 * kNormPasses && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) |
                                                                     reinterpret_cast<uintptr_t>(y)) & 15) == 0;
    if (vec) {
        uint4 xr[kNormPasses], wr[kNormPasses];
        float ss = 0.0f;
#pragma unroll
        for (int p = 0; p < kNormPasses; ++p) {
            const int c8 = tid + p * 256;
            xr[p] = wr[p] = make_uint4(0u, 0u, 0u, 0u);
            if (c8 * 8 < H) {
                xr[p] = *(const uint4 *)(x + base + (size_t)c8 * 8);
                wr[p] = *(const uint4 *)(w + (size_t)c8 * 8);
            }
        }
#pragma unroll
        for (int p = 0; p < kNormPasses; ++p) {
            const uint32_t xw[4] = {xr[p].x, xr[p].y, xr[p].z, xr[p].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float a = h2f((uint16_t)(xw[j] & 0xFFFFu)), c = h2f((uint16_t)(xw[j] >> 16));
                ss += a * a + c * c;
            }
        }
        ss = wave_sum(ss);
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        const float inv = rms_scale((red[0] + red[1] + red[2] + red[3]), 1.0f / (float)H, eps);
#pragma unroll
        for (int p = 0; p < kNormPasses; ++p) {
            const int c8 = tid + p * 256;
            if (c8 * 8 < H) {
                const uint32_t xw[4] = {xr[p].x, xr[p].y, xr[p].z, xr[p].w}, ww[4] = {wr[p].x, wr[p].y, wr[p].z, wr[p].w};
                uint32_t o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint16_t lo = f2h(h2f((uint16_t)(xw[j] & 0xFFFFu)) * inv * h2f((uint16_t)(ww[j] & 0xFFFFu)));
                    const uint16_t hi = f2h(h2f((uint16_t)(xw[j] >> 16)) * inv * h2f((uint16_t)(ww[j] >> 16)));
                    o[j] = (uint32_t)lo | ((uint32_t)hi << 16);
                }
                *(uint4 *)(y + (size_t)b * H + (size_t)c8 * 8) = make_uint4(o[0], o[1], o[2], o[3]);
            }
        }
        return;
    }
    float ss = 0.0f;
    for (int c = tid; c < H; c += 256) {
        const float v = h2f(x[base + c]);
        ss += v * v;
    }
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    const float inv = rms_scale((red[0] + red[1] + red[2] + red[3]), 1.0f / (float)H, eps);
    for (int c = tid; c < H; c += 256) y[(size_t)b * H + c] = f2h(h2f(x[base + c]) * inv * h2f(w[c]));
}

// logits[b0 + b, v] = sum_c xn[b0 + b, c] * W[v, c] for b < NB (at most 8 rows per pass), fp32 accumulate.
// The NB x rows sit in LDS; a wavefront owns one vocabulary row at a time: its lanes stream the row with 16-byte
// loads (8 in flight per lane), take the matching x packets from LDS, and the NB sums are reduced across the
// wavefront at the end of the row.  Persistent grid: wavefront w takes rows w, w + W, w + 2W, ...
template <int NB>
__global__ __launch_bounds__(256) void lm_head_kernel(const uint16_t *__restrict__ xn, const uint16_t *__restrict__ W,
                                                      uint16_t *__restrict__ logits, int b0, int H, int V)
{
    extern __shared__ __align__(16) uint16_t xs[];             // [NB][H]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int packets = H >> 3;
    for (int i = tid; i < NB * packets; i += 256) ((u32x4_t *)xs)[i] = ((const u32x4_t *)(xn + (size_t)b0 * H))[i];
    __syncthreads();
    const int stride = gridDim.x * 4;
    for (int v = blockIdx.x * 4 + wave; v < V; v += stride) {
        const u32x4_t *wrow = (const u32x4_t *)(W + (size_t)v * H);
        float acc[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = 0.0f;
        for (int p0 = 0; p0 < packets; p0 += 512) {
            u32x4_t wv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int p = p0 + j * 64 + lane;
                wv[j] = wrow[min(p, packets - 1)];
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int p = p0 + j * 64 + lane;
                if (p < packets) {
#pragma unroll
                    for (int b = 0; b < NB; ++b) {
                        const u32x4_t xv = ((const u32x4_t *)xs)[b * packets + p];
                        acc[b] = dot2h(wv[j].x, xv.x, acc[b]);
                        acc[b] = dot2h(wv[j].y, xv.y, acc[b]);
                        acc[b] = dot2h(wv[j].z, xv.z, acc[b]);
                        acc[b] = dot2h(wv[j].w, xv.w, acc[b]);
                    }
                }
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float s = wave_sum(acc[b]);
            if (lane == 0) logits[(size_t)(b0 + b) * V + v] = f2h(s);
        }
    }
}

// ids[b] = lowest index among the maxima of logits[b, :] (fp16 values compared as floats); one workgroup per row.
__global__ __launch_bounds__(1024) void argmax_kernel(const uint16_t *__restrict__ logits, int32_t *__restrict__ ids, int V)
{
    __shared__ float bv[16];
    __shared__ int bi[16];
    const uint16_t *row = logits + (size_t)blockIdx.x * V;
    float best = -INFINITY;
    int idx = 0x7FFFFFFF;
    auto take = [&](float v, int c) {
        if (v > best || (v == best && c < idx)) best = v, idx = c;
    };
    if (V % 8 == 0 && (reinterpret_cast<uintptr_t>(logits) & 15) == 0) {
        // 16-byte packets, four of them in flight per thread and round
        const int packets = V >> 3;
        for (int p0 = threadIdx.x; p0 < packets; p0 += 4 * 1024) {
            uint4 raw[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) raw[j] = stream_load((const uint4 *)(row + (size_t)min(p0 + j * 1024, packets - 1) * 8));
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int pk = p0 + j * 1024;
                if (pk < packets) {
                    const uint32_t wv[4] = {raw[j].x, raw[j].y, raw[j].z, raw[j].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        take(h2f((uint16_t)(wv[e] & 0xFFFFu)), pk * 8 + 2 * e);
                        take(h2f((uint16_t)(wv[e] >> 16)), pk * 8 + 2 * e + 1);
                    }
                }
            }
        }
    } else {
        for (int c = threadIdx.x; c < V; c += 1024) take(h2f(row[c]), c);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best, off, kWave);
        const int oi = __shfl_xor(idx, off, kWave);
        if (ov > best || (ov == best && oi < idx)) best = ov, idx = oi;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) bv[wave] = best, bi[wave] = idx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < 16; ++w)
            if (bv[w] > best || (bv[w] == best && bi[w] < idx)) best = bv[w], idx = bi[w];
        ids[blockIdx.x] = idx == 0x7FFFFFFF ? 0 : idx;         // a row of NaNs / -inf only: index 0
    }
}

template <int NB>
hipError_t launch_lm_pass(const uint16_t *xn, const uint16_t *W, uint16_t *logits, int b0, int H, int V, int blocks, hipStream_t stream)
{
    const size_t lds = (size_t)NB * H * sizeof(uint16_t);
    static std::atomic<bool> attr_done{false};   // setting the attribute twice is harmless; the flag only has to be a defined read
    if (!attr_done.load()) {
        if (hipFuncSetAttribute((const void *)lm_head_kernel<NB>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess)
            return hipErrorInvalidValue;
        attr_done.store(true);
    }
    hipLaunchKernelGGL(lm_head_kernel<NB>, dim3(blocks), dim3(256), lds, stream, xn, W, logits, b0, H, V);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_embed(const int32_t *ids, const uint16_t *E, uint16_t *x, int n, int H, int V, uint32_t *err, hipStream_t stream)
{
    hipLaunchKernelGGL(embed_kernel, dim3(n), dim3(256), 0, stream, ids, E, x, H, V, err);
    return hipGetLastError();
}

hipError_t launch_final_norm(const uint16_t *x, const uint16_t *w, uint16_t *y, const SeqTable &st, int H, float eps, hipStream_t stream)
{
    hipLaunchKernelGGL(final_norm_kernel, dim3(st.B), dim3(256), 0, stream, x, w, y, st, H, eps);
    return hipGetLastError();
}

// rows per pass: as many as fit 144 KB of LDS, at most 8
int lm_head_rows_per_pass(int H)
{
    int nb = (144 * 1024) / (2 * H);
    return nb > 8 ? 8 : (nb < 1 ? 1 : nb);
}

hipError_t launch_lm_head(const uint16_t *xn, const uint16_t *W, uint16_t *logits, int B, int H, int V, int n_cus, hipStream_t stream)
{
    const int per = lm_head_rows_per_pass(H);
    for (int b0 = 0; b0 < B;) {
        const int left = B - b0;
        // passes of 8, 4, 2, 1 rows (each instantiation is its own kernel; the remainder is split in powers of two)
        int nb = left >= 8 && per >= 8 ? 8 : left >= 4 && per >= 4 ? 4 : left >= 2 && per >= 2 ? 2 : 1;
        const size_t lds = (size_t)nb * H * 2;
        int per_cu = (int)((150 * 1024) / (lds > 0 ? lds : 1));
        per_cu = per_cu > 8 ? 8 : (per_cu < 1 ? 1 : per_cu);
        int blocks = n_cus * per_cu;
        if (blocks * 4 > V) blocks = (V + 3) / 4;
        hipError_t e;
        switch (nb) {
        case 8: e = launch_lm_pass<8>(xn, W, logits, b0, H, V, blocks, stream); break;
        case 4: e = launch_lm_pass<4>(xn, W, logits, b0, H, V, blocks, stream); break;
        case 2: e = launch_lm_pass<2>(xn, W, logits, b0, H, V, blocks, stream); break;
        default: e = launch_lm_pass<1>(xn, W, logits, b0, H, V, blocks, stream); break;
        }
        if (e != hipSuccess) return e;
        b0 += nb;
    }
    return hipSuccess;
}

hipError_t launch_argmax(const uint16_t *logits, int32_t *ids, int B, int V, hipStream_t stream)
{
    hipLaunchKernelGGL(argmax_kernel, dim3(B), dim3(1024), 0, stream, logits, ids, V);
    return hipGetLastError();
}

}  // namespace relax
