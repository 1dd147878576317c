// Fused int4-decode matrix-vector kernel: out[i,r] = sum_c x[i,c] * (u(r,c) - 8) * s[r, c/32].
//
// The paper's point for this operator (Relax, Sec. 4.2 decode_q4 case study; Sec. 5.1) is that
// the custom 4-bit decode must fuse into the consuming matmul and that batch-1 decoding is served
// by a dedicated matrix-vector program.  On MI355X this kernel is bound by HBM: every packed
// weight byte is read exactly once, straight from global memory into registers with 16-byte loads
// (one quantisation group per lane per load, 1 KB contiguous per wavefront), decoded in registers
// and contracted with the x row held in LDS.  Producer/consumer steps of the layer are fused as
// a prologue (RMSNorm of the x row) and an epilogue (rotary embedding + KV append, residual add,
// SwiGLU), so a decode layer is a handful of launches and no intermediate makes a round trip
// through memory in fp16 more than once.
//
// Decode trick of the fast path (k % 32 == 0, rows 16-byte aligned): or-ing a nibble into the
// mantissa of fp16 1024.0 gives 1024+u (nibble in bits 0..3) or 1024+16u (bits 4..7) without any
// integer->float conversion; v_dot2_f32_f16 multiplies two such values with two x values and
// accumulates in fp32.  The offsets are removed per group with two precomputed sums of x:
//   sum x (u-8) = [sum_A x (1024+u)] + [sum_B x (1024+16u)]/16 - (1032 sum_A x + 72 sum_B x).
// Every quantity is an exact small multiple of the inputs, so integer-valued test cases stay exact.
#include "relax_common.h"

namespace relax {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

__device__ inline float dot2(uint32_t a_bits, uint32_t b_bits, float acc)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a_bits), __builtin_bit_cast(half2_t, b_bits), acc, false);
}

// position of element e (0..7) of a word inside the staged 8-element x packet [x0 x4 x1 x5 x2 x6 x3 x7]
__device__ inline int packet_pos(int e) { return ((e & 3) << 1) | (e >> 2); }

// LDS offset (in halfs) of x element c in the fast-path layout: [chunk of 2048][word j of the group][lane][8]
__device__ inline int fast_off(int c)
{
    int chunk = c >> 11, lane = (c & 2047) >> 5, j = (c & 31) >> 3, e = c & 7;
    return ((((chunk << 2) + j) << 6) + lane) * 8 + packet_pos(e);
}

template <int EPI>
__device__ inline int unit_count(const GemvArgs &a)
{
    if (EPI == EPI_SWIGLU) return a.m / 2;
    return (a.m + 1) / 2;
}

// unit u -> the two matrix rows whose results the epilogue consumes together
template <int EPI>
__device__ inline void unit_rows(const GemvArgs &a, int u, int &ra, int &rb)
{
    if (EPI == EPI_SWIGLU) {
        ra = u;
        rb = u + a.m / 2;
    } else if (EPI == EPI_ROPE_KV) {
        int hd2 = a.d >> 1, nqk = (a.h + a.g) * hd2;
        if (u < nqk) {
            int j = u / hd2, t = u - j * hd2;
            ra = j * a.d + t;
            rb = ra + hd2;
        } else {
            ra = (a.h + a.g) * a.d + 2 * (u - nqk);
            rb = ra + 1;
        }
    } else {
        ra = 2 * u;
        rb = min(2 * u + 1, a.m - 1);
    }
}

template <int EPI>
__device__ inline void epilogue(const GemvArgs &a, int i, const RowInfo &ri, int u, float va, float vb)
{
    int ra, rb;
    unit_rows<EPI>(a, u, ra, rb);
    size_t base = (size_t)i * a.m;
    if (EPI == EPI_F16) {
        a.out_f16[base + ra] = f2h(va);
        if (2 * u + 1 < a.m) a.out_f16[base + rb] = f2h(vb);
    } else if (EPI == EPI_RESID_F32) {
        const uint16_t *xr = (const uint16_t *)a.resid;
        a.out_f32[base + ra] = h2f(xr[base + ra]) + va;
        if (2 * u + 1 < a.m) a.out_f32[base + rb] = h2f(xr[base + rb]) + vb;
    } else if (EPI == EPI_RESID_F16) {
        const float *xr = (const float *)a.resid;
        a.out_f16[base + ra] = f2h(xr[base + ra] + va);
        if (2 * u + 1 < a.m) a.out_f16[base + rb] = f2h(xr[base + rb] + vb);
    } else if (EPI == EPI_SWIGLU) {
        float act = va / (1.0f + expf(-va)) * vb;
        a.out_f16[(size_t)i * (a.m / 2) + u] = f2h(act);
    } else {  // EPI_ROPE_KV
        int hd2 = a.d >> 1, nqk = (a.h + a.g) * hd2;
        size_t tok = ((size_t)ri.slot * a.kv_capacity + ri.pos) * (size_t)(a.g * a.d);
        if (u < nqk) {
            int j = u / hd2, t = u - j * hd2;
            float c = a.rope[((size_t)ri.pos * hd2 + t) * 2], s = a.rope[((size_t)ri.pos * hd2 + t) * 2 + 1];
            float oa = va * c - vb * s, ob = va * s + vb * c;
            if (j < a.h) {
                size_t at = (size_t)i * (a.h * a.d) + (size_t)j * a.d + t;
                a.out_f16[at] = f2h(oa);
                a.out_f16[at + hd2] = f2h(ob);
            } else {
                size_t at = tok + (size_t)(j - a.h) * a.d + t;
                a.kcache[at] = f2h(oa);
                a.kcache[at + hd2] = f2h(ob);
            }
        } else {
            size_t at = tok + 2 * (size_t)(u - nqk);
            a.vcache[at] = f2h(va);
            a.vcache[at + 1] = f2h(vb);
        }
    }
}

template <int XMODE>
__device__ inline float load_x(const GemvArgs &a, size_t idx)
{
    if (XMODE == X_F32_NORM) return ((const float *)a.x)[idx];
    return h2f(((const uint16_t *)a.x)[idx]);
}

template <int XMODE, int EPI, bool FAST>
__global__ __launch_bounds__(512) void gemv_q4_kernel(GemvArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red[8];
    const int k = a.k, G = (k + kGroup - 1) / kGroup, kw = k >> 3;
    const int kpad = FAST ? ((k + 2047) >> 11) << 11 : k;
    uint16_t *xs = (uint16_t *)smem;
    float *corr = (float *)(smem + (size_t)kpad * 2);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
    const int i = blockIdx.y;                       // row of x served by this block
    const size_t xbase = (size_t)i * k;

    // ---- prologue: stage the (optionally RMS-normalised) x row in LDS as fp16 ----------------
    float inv = 1.0f;
    if (XMODE != X_F16) {
        float ss = 0.0f;
        for (int c = tid; c < k; c += blockDim.x) {
            float v = load_x<XMODE>(a, xbase + c);
            ss += v * v;
        }
        ss = wave_sum(ss);
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        float tot = 0.0f;
        for (int w = 0; w < nwaves; ++w) tot += red[w];
        inv = 1.0f / sqrtf(tot / (float)k + a.eps);
    }
    for (int c = tid; c < kpad; c += blockDim.x) {
        float v = 0.0f;
        if (c < k) {
            v = load_x<XMODE>(a, xbase + c);
            if (XMODE != X_F16) v = v * inv * h2f(a.norm_w[c]);
        }
        xs[FAST ? fast_off(c) : c] = f2h(v);
    }
    __syncthreads();
    if (FAST) {
        for (int gi = tid; gi < G; gi += blockDim.x) {
            int chunk = gi >> 6, ln = gi & 63;
            float sa = 0.0f, sb = 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint16_t *p = xs + ((((chunk << 2) + j) << 6) + ln) * 8;
                sa += h2f(p[0]) + h2f(p[1]) + h2f(p[4]) + h2f(p[5]);
                sb += h2f(p[2]) + h2f(p[3]) + h2f(p[6]) + h2f(p[7]);
            }
            corr[gi] = 1032.0f * sa + 72.0f * sb;
        }
        __syncthreads();
    }

    RowInfo ri = {0, 0, 0};
    if (EPI == EPI_ROPE_KV) ri = row_info(a.seqs, i);

    // ---- main loop: each wavefront owns two units (four matrix rows) per trip ----------------
    const int U = unit_count<EPI>(a);
    const int nchunks = (G + 63) >> 6;
    for (int u0 = (blockIdx.x * nwaves + wave) * 2; u0 < U; u0 += gridDim.x * nwaves * 2) {
        int rows[4];
        unit_rows<EPI>(a, u0, rows[0], rows[1]);
        const bool second = (u0 + 1 < U);
        unit_rows<EPI>(a, second ? u0 + 1 : u0, rows[2], rows[3]);
        float tot[4] = {0.0f, 0.0f, 0.0f, 0.0f};

        if (FAST) {
            for (int chunk = 0; chunk < nchunks; ++chunk) {
                const int gi = (chunk << 6) + lane;
                if (gi < G) {
                    uint4 xv[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        xv[j] = *(const uint4 *)(xs + ((((chunk << 2) + j) << 6) + lane) * 8);
                    const float cr = corr[gi];
                    uint4 wv[4];
                    float sc[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        wv[r] = *(const uint4 *)(a.q + (size_t)rows[r] * kw + (size_t)gi * 4);
                        sc[r] = h2f(a.s[(size_t)rows[r] * G + gi]);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const uint32_t ww[4] = {wv[r].x, wv[r].y, wv[r].z, wv[r].w};
                        float accA = 0.0f, accB = 0.0f;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const uint32_t w = ww[j], w8 = w >> 8;
                            const uint32_t xw[4] = {xv[j].x, xv[j].y, xv[j].z, xv[j].w};
                            accA = dot2((w & 0x000F000Fu) | 0x64006400u, xw[0], accA);
                            accB = dot2((w & 0x00F000F0u) | 0x64006400u, xw[1], accB);
                            accA = dot2((w8 & 0x000F000Fu) | 0x64006400u, xw[2], accA);
                            accB = dot2((w8 & 0x00F000F0u) | 0x64006400u, xw[3], accB);
                        }
                        tot[r] += sc[r] * (accA + accB * 0.0625f - cr);
                    }
                }
            }
        } else {
            // any k % 8 == 0 (short last group, unaligned rows): the definition, word by word
            for (int widx = lane; widx < kw; widx += kWave) {
                float xv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) xv[e] = h2f(xs[widx * 8 + e]);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const uint32_t word = a.q[(size_t)rows[r] * kw + widx];
                    const float sc = h2f(a.s[(size_t)rows[r] * G + (widx >> 2)]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) tot[r] += xv[e] * ((float)decode_code(word, e) * sc);
                }
            }
        }

#pragma unroll
        for (int r = 0; r < 4; ++r) tot[r] = wave_sum(tot[r]);
        if (lane == 0) {
            epilogue<EPI>(a, i, ri, u0, tot[0], tot[1]);
            if (second) epilogue<EPI>(a, i, ri, u0 + 1, tot[2], tot[3]);
        }
    }
}

template <int XMODE, int EPI>
static hipError_t launch_t(const GemvArgs &a, hipStream_t stream)
{
    const int k = a.k, G = groups_of(k);
    const bool fast = (k % kGroup == 0) && ((k / 8) % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.q) & 15) == 0);
    const int threads = 512, nwaves = threads / kWave;
    int U = (EPI == EPI_SWIGLU) ? a.m / 2 : (a.m + 1) / 2;
    int gx = (U + 2 * nwaves - 1) / (2 * nwaves);
    if (gx > 1024) gx = 1024;
    if (gx < 1) gx = 1;
    dim3 grid(gx, a.n), block(threads);
    if (fast) {
        size_t lds = (size_t)((k + 2047) / 2048) * 2048 * 2 + (size_t)G * 4;
        hipLaunchKernelGGL((gemv_q4_kernel<XMODE, EPI, true>), grid, block, lds, stream, a);
    } else {
        size_t lds = (size_t)k * 2;
        hipLaunchKernelGGL((gemv_q4_kernel<XMODE, EPI, false>), grid, block, lds, stream, a);
    }
    return hipGetLastError();
}

hipError_t launch_gemv(const GemvArgs &a, int xmode, int epi, hipStream_t stream)
{
    if (xmode == X_F16 && epi == EPI_F16) return launch_t<X_F16, EPI_F16>(a, stream);
    if (xmode == X_F16_NORM && epi == EPI_ROPE_KV) return launch_t<X_F16_NORM, EPI_ROPE_KV>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F32) return launch_t<X_F16, EPI_RESID_F32>(a, stream);
    if (xmode == X_F32_NORM && epi == EPI_SWIGLU) return launch_t<X_F32_NORM, EPI_SWIGLU>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F16) return launch_t<X_F16, EPI_RESID_F16>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace relax
