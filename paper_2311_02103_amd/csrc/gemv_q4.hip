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
#include <algorithm>
#include <cstdlib>

#include "q4_device.h"

namespace relax {

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
    const int k = a.k, G = (k + kGroup - 1) / kGroup, kw = k >> 3, SG = scales_per_row(k, a.gshift);
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
        inv = rms_scale(tot, 1.0f / (float)k, a.eps);
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
        for (int gi = tid; gi < G; gi += blockDim.x) corr[gi] = group_corr(xs, gi);
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
                        wv[r] = stream_load((const uint4 *)(a.q + (size_t)rows[r] * kw + (size_t)gi * 4));
                        sc[r] = h2f(a.s[(size_t)rows[r] * SG + (gi >> a.gshift)]);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) tot[r] += sc[r] * group_dot(wv[r], xv, cr);
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
                    const float sc = h2f(a.s[(size_t)rows[r] * SG + ((widx >> 2) >> a.gshift)]);
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

// ---- streaming kernel for the fast layout (k % 32 == 0, 16-byte aligned rows) -----------------------------------------
//
// Persistent shape: a few workgroups per CU, six wavefronts each; every wavefront walks tiles of four matrix
// rows (two units the epilogue consumes together) in trips of 4 rows x 2 chunks of 2048 columns = 8 KB, with
// two trips in flight (double buffer, branch-free so that consuming one trip never waits for the next one).
// The first two trips are requested BEFORE the x row is staged -- weights do not depend on x -- and the
// workgroup barriers of the staging fence LDS only, so those loads stay in flight across them.  Sums of a
// tile go to LDS; after the loop lane j finishes the wavefront's j-th tile (loads and stores of the
// epilogue never interleave with the weight stream).
constexpr int kSThreads = 256, kSWaves = kSThreads / kWave, kSMaxTiles = 16;

template <int EPI>
__device__ __forceinline__ void stream_tile_rows(const GemvArgs &a, int tile, int *rows)
{
    if (EPI == EPI_ROPE_KV) {
        const int d4 = a.d >> 2, nqk = (a.h + a.g) * d4;
        if (tile < nqk) {
            const int j = tile / d4, t = (tile - j * d4) * 2;
            rows[0] = j * a.d + t, rows[1] = rows[0] + (a.d >> 1), rows[2] = rows[0] + 1, rows[3] = rows[1] + 1;
        } else {
            rows[0] = (a.h + a.g) * a.d + 4 * (tile - nqk);
            rows[1] = rows[0] + 1, rows[2] = rows[0] + 2, rows[3] = rows[0] + 3;
        }
    } else if (EPI == EPI_SWIGLU) {
        const int F = a.m >> 1;
        rows[0] = 2 * tile, rows[1] = rows[0] + F, rows[2] = rows[0] + 1, rows[3] = rows[1] + 1;
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) rows[r] = min(4 * tile + r, a.m - 1);
    }
}

template <int EPI>
__device__ __forceinline__ void stream_epilogue(const GemvArgs &a, int i, const RowInfo &ri, int tile, const float *v)
{
    const size_t base = (size_t)i * a.m;
    if (EPI == EPI_F16 || EPI == EPI_RESID_F32 || EPI == EPI_RESID_F16) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * tile + r;
            if (row < a.m) {
                if (EPI == EPI_F16) a.out_f16[base + row] = f2h(v[r]);
                else if (EPI == EPI_RESID_F32) a.out_f32[base + row] = h2f(((const uint16_t *)a.resid)[base + row]) + v[r];
                else a.out_f16[base + row] = f2h(((const float *)a.resid)[base + row] + v[r]);
            }
        }
    } else if (EPI == EPI_SWIGLU) {
        const int F = a.m >> 1;
        uint16_t *dst = a.out_f16 + (size_t)i * F + 2 * tile;
        dst[0] = f2h(v[0] / (1.0f + expf(-v[0])) * v[1]);
        dst[1] = f2h(v[2] / (1.0f + expf(-v[2])) * v[3]);
    } else {  // EPI_ROPE_KV
        const int d4 = a.d >> 2, hd2 = a.d >> 1, nqk = (a.h + a.g) * d4;
        const size_t tok = ((size_t)ri.slot * a.kv_capacity + ri.pos) * (size_t)(a.g * a.d);
        if (tile < nqk) {
            const int j = tile / d4, t = (tile - j * d4) * 2;
            const float4 cs = *(const float4 *)(a.rope + ((size_t)ri.pos * hd2 + t) * 2);       // cos_t sin_t cos_t+1 sin_t+1
            const float p0 = v[0] * cs.x - v[1] * cs.y, q0 = v[0] * cs.y + v[1] * cs.x;
            const float p1 = v[2] * cs.z - v[3] * cs.w, q1 = v[2] * cs.w + v[3] * cs.z;
            uint16_t *dst = (j < a.h) ? a.out_f16 + (size_t)i * (a.h * a.d) + (size_t)j * a.d + t
                                      : a.kcache + tok + (size_t)(j - a.h) * a.d + t;
            dst[0] = f2h(p0), dst[1] = f2h(p1), dst[hd2] = f2h(q0), dst[hd2 + 1] = f2h(q1);
        } else {
            uint16_t *dst = a.vcache + tok + 4 * (size_t)(tile - nqk);
#pragma unroll
            for (int r = 0; r < 4; ++r) dst[r] = f2h(v[r]);
        }
    }
}

template <int XMODE, int EPI, int PX>
__global__ __launch_bounds__(kSThreads) void gemv_q4_stream_kernel(GemvArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ float red[kSWaves];
    const int k = a.k, G = k >> 5, nchunks = (k + 2047) >> 11, kpad = nchunks << 11;
    uint16_t *xs = (uint16_t *)smem;
    float *corr = (float *)(smem + (size_t)kpad * 2);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float *res = corr + ((G + 63) & ~63) + wave * (kSMaxTiles * 4);
    const int i = blockIdx.y;
    const DLMat M = {a.q, a.s, a.m, a.k, a.gshift};
    const int ntiles = (EPI == EPI_ROPE_KV || EPI == EPI_SWIGLU) ? (a.m >> 2) : ((a.m + 3) >> 2);
    const int nsub = (nchunks + 1) >> 1;
    const int W = gridDim.x * kSWaves, wave_global = blockIdx.x * kSWaves + wave;
    const int mine = wave_global < ntiles ? (ntiles - wave_global + W - 1) / W : 0;
    const int nsu = mine * nsub;

    auto target = [&](int su, int *rows, int &chunk0) {
        const bool live = su < nsu;
        const int j = su / nsub, sub = su - j * nsub;
        stream_tile_rows<EPI>(a, live ? wave_global + j * W : 0, rows);
        chunk0 = live ? sub * 2 : 0;
    };
    // ---- loads in the order they are needed: memory operations of a wavefront complete in order, so the x row (and
    //      the norm weights) go out first and the two weight trips right behind them -------------------------------
    const size_t xbase = (size_t)i * k;
    constexpr int PN = 4;                   // passes of 256 threads x 8 elements: PN covers 8192 (norm modes), PX the plain row
    float vals[XMODE != X_F16 ? PN : 1][8];
    uint4 wnr[XMODE != X_F16 ? PN : 1];
    uint4 xraw[XMODE == X_F16 ? PX : 1];
    if (XMODE != X_F16) {
#pragma unroll
        for (int p = 0; p < PN; ++p) {
            const int c8 = min(tid + p * kSThreads, (k >> 3) - 1);
            if (XMODE == X_F32_NORM) {
                const float4 lo = *(const float4 *)((const float *)a.x + xbase + c8 * 8), hi = *(const float4 *)((const float *)a.x + xbase + c8 * 8 + 4);
                vals[p][0] = lo.x, vals[p][1] = lo.y, vals[p][2] = lo.z, vals[p][3] = lo.w;
                vals[p][4] = hi.x, vals[p][5] = hi.y, vals[p][6] = hi.z, vals[p][7] = hi.w;
            } else {
                const uint4 raw = *(const uint4 *)((const uint16_t *)a.x + xbase + c8 * 8);
                const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int j = 0; j < 4; ++j) vals[p][2 * j] = h2f((uint16_t)(w[j] & 0xFFFFu)), vals[p][2 * j + 1] = h2f((uint16_t)(w[j] >> 16));
            }
            wnr[p] = *(const uint4 *)(a.norm_w + c8 * 8);
        }
    } else {
#pragma unroll
        for (int p = 0; p < PX; ++p) {
            const int c8 = min(tid + p * kSThreads, (k >> 3) - 1);
            xraw[p] = *(const uint4 *)((const uint16_t *)a.x + xbase + c8 * 8);
        }
    }
    Slot s0, s1;
    {
        int rows[4], chunk0;
        target(0, rows, chunk0);
        slot_load(s0, M, rows, chunk0, 0, lane);
        target(1, rows, chunk0);
        slot_load(s1, M, rows, chunk0, 0, lane);
    }

    // ---- stage the (optionally RMS-normalised) x row in LDS as fp16 in the packet order [x0 x4 x1 x5 x2 x6 x3 x7] ----
    auto put8 = [&](int c8, const float *y) {
        const uint32_t o0 = (uint32_t)f2h(y[0]) | ((uint32_t)f2h(y[4]) << 16), o1 = (uint32_t)f2h(y[1]) | ((uint32_t)f2h(y[5]) << 16);
        const uint32_t o2 = (uint32_t)f2h(y[2]) | ((uint32_t)f2h(y[6]) << 16), o3 = (uint32_t)f2h(y[3]) | ((uint32_t)f2h(y[7]) << 16);
        *(uint4 *)(xs + fast_off(c8 * 8)) = make_uint4(o0, o1, o2, o3);
    };
    if (XMODE != X_F16) {
        float ss = 0.0f;
#pragma unroll
        for (int p = 0; p < PN; ++p)
            if ((tid + p * kSThreads) * 8 < k) {
#pragma unroll
                for (int e = 0; e < 8; ++e) ss += vals[p][e] * vals[p][e];
            }
        ss = wave_sum(ss);
        if (lane == 0) red[wave] = ss;
        wg_barrier();
        float tot = 0.0f;
#pragma unroll
        for (int w = 0; w < kSWaves; ++w) tot += red[w];
        const float inv = rms_scale(tot, 1.0f / (float)k, a.eps);
#pragma unroll
        for (int p = 0; p < PN; ++p) {
            const int c8 = tid + p * kSThreads;
            if (c8 * 8 < kpad) {
                const uint32_t w[4] = {wnr[p].x, wnr[p].y, wnr[p].z, wnr[p].w};
                float y[8];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    y[2 * j] = c8 * 8 < k ? vals[p][2 * j] * inv * h2f((uint16_t)(w[j] & 0xFFFFu)) : 0.0f;
                    y[2 * j + 1] = c8 * 8 < k ? vals[p][2 * j + 1] * inv * h2f((uint16_t)(w[j] >> 16)) : 0.0f;
                }
                put8(c8, y);
            }
        }
    } else {
#pragma unroll
        for (int p = 0; p < PX; ++p) {
            const int c8 = tid + p * kSThreads;
            if (c8 * 8 < kpad) {
                const uint32_t w[4] = {xraw[p].x, xraw[p].y, xraw[p].z, xraw[p].w};
                float y[8];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    y[2 * j] = c8 * 8 < k ? h2f((uint16_t)(w[j] & 0xFFFFu)) : 0.0f;
                    y[2 * j + 1] = c8 * 8 < k ? h2f((uint16_t)(w[j] >> 16)) : 0.0f;
                }
                put8(c8, y);
            }
        }
    }
    wg_barrier();
    for (int gi = tid; gi < G; gi += kSThreads) corr[gi] = group_corr(xs, gi);
    wg_barrier();

    RowInfo ri = {0, 0, 0};
    if (EPI == EPI_ROPE_KV) ri = row_info(a.seqs, i);

    // ---- trips ------------------------------------------------------------------------------------------------
    float acc8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc8[e] = 0.0f;
    auto trip = [&](Slot &s, int su, bool prefetch) {
        const int j = su / nsub, sub = su - j * nsub;
        slot_consume(s, M, xs, corr, sub * 2, 0, lane, su < nsu, acc8);
        if (prefetch) {                                            // compile-time constant at both call sites
            int rows[4], chunk0;
            target(su + 2, rows, chunk0);
            slot_load(s, M, rows, chunk0, 0, lane);
        }
        if (su < nsu && sub == nsub - 1) {
            float v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = wave_sum(acc8[r] + acc8[r + 4]);
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) res[j * 4 + r] = v[r];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc8[e] = 0.0f;
        }
    };
    // The last two trips are peeled off the loop and request nothing: a wavefront does not retire before its
    // outstanding loads have returned, so prefetching past the end would add a memory round trip to every launch.
    const int nsu_even = (nsu + 1) & ~1;
    int su = 0;
#pragma unroll 1
    for (; su + 2 < nsu_even; su += 2) {
        trip(s0, su, true);
        trip(s1, su + 1, true);
    }
    trip(s0, su, false);
    trip(s1, su + 1, false);
    if (lane < mine) {
        float v[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = res[lane * 4 + r];
        stream_epilogue<EPI>(a, i, ri, wave_global + lane * W, v);
    }
}

template <int XMODE, int EPI>
static hipError_t launch_t(const GemvArgs &a, hipStream_t stream)
{
    // rows of 12289 .. 28672 columns behind a plain prologue, and from two rows of x on rows of 8193 columns up (several rows of x per pass)
    if (gemv_long_eligible(a, XMODE, EPI)) return launch_gemv_long(a, EPI, stream);
    if (gemv_reg_eligible(a)) return launch_gemv_reg(a, XMODE, EPI, stream);
    const int k = a.k, G = groups_of(k);
    const bool fast = (k % kGroup == 0) && ((k / 8) % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.q) & 15) == 0) &&
                      ((reinterpret_cast<uintptr_t>(a.x) & 15) == 0) && ((reinterpret_cast<uintptr_t>(a.norm_w) & 15) == 0);
    const int threads = 512, nwaves = threads / kWave;
    int U = (EPI == EPI_SWIGLU) ? a.m / 2 : (a.m + 1) / 2;
    int gx = (U + 2 * nwaves - 1) / (2 * nwaves);
    if (gx > 1024) gx = 1024;
    if (gx < 1) gx = 1;
    dim3 grid(gx, a.n), block(threads);
    if (fast && (XMODE == X_F16 ? k <= 14 * kSThreads * 8 : k <= 4 * kSThreads * 8)) {
        const int ntiles = (EPI == EPI_ROPE_KV || EPI == EPI_SWIGLU) ? a.m / 4 : (a.m + 3) / 4;
        const size_t lds = (size_t)((k + 2047) / 2048) * 2048 * 2 + (size_t)((G + 63) / 64 * 64) * 4 + kSWaves * kSMaxTiles * 4 * 4;
        const bool small_k = k <= 6 * kSThreads * 8;
        auto kern = small_k ? gemv_q4_stream_kernel<XMODE, EPI, 6> : gemv_q4_stream_kernel<XMODE, EPI, 14>;
        // workgroups that are resident at the same time (CUs x occupancy): the grid never exceeds it, so that every
        // workgroup starts at once and each wavefront keeps streaming until its share is done
        static int resident[2] = {0, 0};
        if (resident[small_k] == 0) {
            int dev = 0, cus = 0, occ = 0;
            if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) cus = 256;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kern, kSThreads, 40 * 1024) != hipSuccess || occ < 1) occ = 1;
            resident[small_k] = cus * std::max(1, std::min(occ, 1));       // one workgroup per CU (two measured slower)
        }
        int sgx = std::max(1, resident[small_k] / std::min(a.n, 8));
        sgx = std::min(sgx, (ntiles + kSWaves - 1) / kSWaves);
        sgx = std::max(sgx, (ntiles + kSWaves * kSMaxTiles - 1) / (kSWaves * kSMaxTiles));
        hipLaunchKernelGGL(kern, dim3(sgx, a.n), dim3(kSThreads), lds, stream, a);
    } else {
        size_t lds = (size_t)k * 2;
        hipLaunchKernelGGL((gemv_q4_kernel<XMODE, EPI, false>), grid, block, lds, stream, a);
    }
    return hipGetLastError();
}

hipError_t launch_gemv(const GemvArgs &a, int xmode, int epi, hipStream_t stream)
{
    if (xmode == X_ATTN_MERGE) return launch_gemv_reg(a, xmode, epi, stream);      // only the x-in-registers kernel folds the merge
    if (xmode == X_F16 && epi == EPI_F16) return launch_t<X_F16, EPI_F16>(a, stream);
    if (xmode == X_F16_NORM && epi == EPI_ROPE_KV) return launch_t<X_F16_NORM, EPI_ROPE_KV>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F32) return launch_t<X_F16, EPI_RESID_F32>(a, stream);
    if (xmode == X_F32_NORM && epi == EPI_SWIGLU) return launch_t<X_F32_NORM, EPI_SWIGLU>(a, stream);
    if (xmode == X_F16 && epi == EPI_RESID_F16) return launch_t<X_F16, EPI_RESID_F16>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace relax
