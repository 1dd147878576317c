// Device-side pieces shared by the kernels that stream packed int4 weights: the in-register decode +
// contraction of one quantisation group, the LDS layout of the staged x row, wavefront reductions.
#pragma once

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

// One quantisation group (4 words = 32 codes) against the lane's 32 staged x values:
// returns sum_c x_c * (u_c - 8) given corr = 1032 * sum_A x + 72 * sum_B x of that group.
// (w & 0x000F000F) | 0x64006400 is the fp16 pair (1024+u0, 1024+u4); (w & 0x00F000F0) | 0x64006400 is
// (1024+16 u1, 1024+16 u5); the same masks on w >> 8 give nibbles 2,6 and 3,7.
__device__ inline float group_dot(const uint4 &wq, const uint4 *xv, float corr)
{
    const uint32_t ww[4] = {wq.x, wq.y, wq.z, wq.w};
    float accA = 0.0f, accB = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t w = ww[j], w8 = w >> 8;
        accA = dot2((w & 0x000F000Fu) | 0x64006400u, xv[j].x, accA);
        accB = dot2((w & 0x00F000F0u) | 0x64006400u, xv[j].y, accB);
        accA = dot2((w8 & 0x000F000Fu) | 0x64006400u, xv[j].z, accA);
        accB = dot2((w8 & 0x00F000F0u) | 0x64006400u, xv[j].w, accB);
    }
    return accA + accB * 0.0625f - corr;
}

// per-group offset term of the staged row: 1032 * (x0+x4+x2+x6 over the 4 words) + 72 * (x1+x5+x3+x7 ...)
__device__ inline float group_corr(const uint16_t *xs, int gi)
{
    const int chunk = gi >> 6, ln = gi & 63;
    float sa = 0.0f, sb = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint16_t *p = xs + ((((chunk << 2) + j) << 6) + ln) * 8;
        sa += h2f(p[0]) + h2f(p[1]) + h2f(p[4]) + h2f(p[5]);
        sb += h2f(p[2]) + h2f(p[3]) + h2f(p[6]) + h2f(p[7]);
    }
    return 1032.0f * sa + 72.0f * sb;
}

// Workgroup barrier that orders LDS only: outstanding global loads (the weight trips) stay in flight across it.
__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// eight 16-byte weight loads + eight scales of one wavefront trip.  A trip covers either 4 rows x 2 chunks
// of 2048 columns (mode 0: rotary / SwiGLU steps, whose epilogues need four rows) or 2 rows x 4 chunks
// (mode 1: the residual steps).  Entry e of the slot is (row r, chunk c) with e = c * rows + r.
struct Slot {
    uint4 w[8];
    uint16_t sc[8];
};

// Everything here is branch-free and shared by all steps (ONE copy of the trip code in the kernel: the whole
// kernel has to fit the instruction cache): a trip is ALWAYS 16 loads -- lanes or whole trips that have nothing
// to fetch re-read a clamped, cache-resident address and contribute with scale 0 -- so the instruction stream,
// and with it the compiler's count of loads in flight, is static and consuming one trip never waits for the
// trip requested after it.
__device__ __forceinline__ void slot_load(Slot &s, const DLMat &M, const int *rows, int chunk0, int mode, int lane)
{
    const int G = M.k >> 5, kw = M.k >> 3, SG = scales_per_row(M.k, M.gshift);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int row = mode ? rows[e & 1] : rows[e & 3], c = mode ? (e >> 1) : (e >> 2);    // static indices only
        const int gi = min(((chunk0 + c) << 6) + lane, G - 1);
        s.w[e] = *(const uint4 *)(M.q + (size_t)row * kw + (size_t)gi * 4);
        s.sc[e] = M.s[(size_t)row * SG + (gi >> M.gshift)];
    }
}

__device__ __forceinline__ void slot_consume(const Slot &s, const DLMat &M, const uint16_t *xs, const float *corr, int chunk0,
                                             int mode, int lane, bool live, float *acc8)
{
    if (!live) return;                                             // wave-uniform: a dead trip only keeps the load pattern static
    const int G = M.k >> 5, last_chunk = (G - 1) >> 6;
    uint4 xv[4];
    float cr = 0.0f;
    bool on = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if ((e & 1) == 0) {                                        // the chunk can only change on even entries
            const int c = mode ? (e >> 1) : (e >> 2);
            const int gi = ((chunk0 + c) << 6) + lane;
            const int chunk = min(chunk0 + c, last_chunk);         // keeps the LDS reads inside the staged row
            on = live && gi < G;
#pragma unroll
            for (int j = 0; j < 4; ++j) xv[j] = *(const uint4 *)(xs + ((((chunk << 2) + j) << 6) + lane) * 8);
            cr = corr[min(gi, G - 1)];
        }
        acc8[e] += (on ? h2f(s.sc[e]) : 0.0f) * group_dot(s.w[e], xv, cr);
    }
}

}  // namespace relax
