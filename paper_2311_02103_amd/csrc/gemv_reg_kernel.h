// Batch-1 matrix-vector kernel with the x row in registers (Relax, Sec. 4.2 decode_q4 case study: the 4-bit decode
// fused into the consuming matmul; Sec. 5.1: batch-1 decoding served by a dedicated matrix-vector program).
//
// The kernel is bound by HBM, and at the sizes of one decoder layer a launch lasts ~10 us, so what counts besides
// the stream itself is (a) how few vector instructions a weight costs -- one wavefront per SIMD leaves nothing to
// hide them behind -- and (b) how short the x-dependent prologue and the tail are:
//   * one workgroup of four wavefronts per CU; a wavefront walks the rows of its units (row pairs the epilogue
//     consumes together) in slots of one or two rows, two slots in flight, 16-byte loads (one quantisation group per
//     lane and load, 1 KB contiguous per wavefront).  Small slots: what a wavefront still has to compute when its last
//     byte arrives is the arithmetic of the slots in flight;
//   * the first slots are requested before anything that depends on x; x is staged once per workgroup through LDS
//     (RMSNorm folded in) and then lives in registers in the packet order of the decode: lane l owns groups
//     l, l + 64, ... of the row, exactly the groups its weight loads bring, so the loop touches no LDS;
//   * decode: (w & 0x000F000F) | 0x6400 6400 is the fp16 pair (1024 + u0, 1024 + u4) in one v_and_or_b32, the other
//     masks give (1024 + 16 u1, 1024 + 16 u5) and, on w >> 8, nibbles 2,6 and 3,7; v_dot2_f32_f16 contracts a pair with
//     two x values in fp32 and the offsets leave per group through 1032 sum_A x + 72 sum_B x (exact arithmetic on
//     integer-valued inputs);
//   * the row sums of a slot are reduced together with DPP row operations (for two rows a transposing reduction;
//     2 LDS-crossbar exchanges per slot instead of 6 per row);
//   * inputs of the epilogue (residual values, rotary table entries) are fetched at the very start, results are
//     parked in LDS and lane j finishes the wavefront's j-th unit after the stream has drained, so no load of the
//     epilogue ever sits between weight loads (memory operations of a wavefront return in order).
//
// This header holds the kernel and its launch templates; the launchers of the three weight streams (4-bit, plain fp16, native
// 3-bit) are translation units of their own (gemv_q4_reg.hip, gemv_reg_f16.hip, gemv_reg_q3.hip), each a code object of
// its own, compiled side by side.
#pragma once
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "q4_device.h"

namespace relax {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kRThreads = 256, kRWaves = kRThreads / kWave;
constexpr int kRMaxUnits = 64;            // units per wavefront: lane j finishes unit j

// (w & mask) | bits as one VALU op (mask from a scalar register, bits from a vector register)
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t bits)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(bits));
    return r;
}

// sum_c x_c (u_c - 8) of one group: wq = its four words, xv = the lane's 32 x values in packet order
// ([x0 x4 x1 x5 x2 x6 x3 x7] per word), corr = 1032 sum_A x + 72 sum_B x
__device__ __forceinline__ float group_dot_r(const u32x4_t &wq, const u32x4_t *xv, float corr)
{
    const uint32_t base = 0x64006400u;
    float accA = 0.0f, accB = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t w = wq[j], w8 = w >> 8;
        accA = dot2(and_or(w, 0x000F000Fu, base), xv[j].x, accA);
        accB = dot2(and_or(w, 0x00F000F0u, base), xv[j].y, accB);
        accA = dot2(and_or(w8, 0x000F000Fu, base), xv[j].z, accA);
        accB = dot2(and_or(w8, 0x00F000F0u, base), xv[j].w, accB);
    }
    return accA + accB * 0.0625f - corr;
}

// value of another lane through a DPP control word (all lanes active, full row and bank masks)
template <int CTRL>
__device__ __forceinline__ float dpp(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
constexpr int kQuadXor1 = 0xB1, kQuadXor2 = 0x4E, kRowRor4 = 0x124, kRowRor8 = 0x128;

// one partial sum -> every lane holds the total
__device__ __forceinline__ float reduce1(float v)
{
    float r = v + dpp<kQuadXor1>(v);
    r += dpp<kQuadXor2>(r);
    r += dpp<kRowRor4>(r);
    r += dpp<kRowRor8>(r);
    r = xor16_sum(r);
    r = xor32_sum(r);
    return r;
}
// two partial sums -> lane l holds the total of row l & 1
__device__ __forceinline__ float reduce2(float v0, float v1, int lane)
{
    const bool odd = lane & 1;
    float r = (odd ? v1 : v0) + dpp<kQuadXor1>(odd ? v0 : v1);
    r += dpp<kQuadXor2>(r);
    r += dpp<kRowRor4>(r);
    r += dpp<kRowRor8>(r);
    r = xor16_sum(r);
    r = xor32_sum(r);
    return r;
}

// u / hd2 for the rotary row mapping: a shift when half the head dimension is a power of two (the branch is uniform
// and holds no load)
__device__ __forceinline__ int div_half_dim(int u, int hd2)
{
    if ((hd2 & (hd2 - 1)) == 0) return u >> (31 - __builtin_clz(hd2));
    return u / hd2;
}

template <int EPI>
__device__ __forceinline__ int unit_count_r(const GemvArgs &a)
{
    return (EPI == EPI_SWIGLU || EPI == EPI_ROPE_KV) ? a.m / 2 : (a.m + 1) / 2;
}

// unit u -> the two matrix rows whose results the epilogue consumes together
template <int EPI>
__device__ __forceinline__ void unit_rows_r(const GemvArgs &a, int u, int &ra, int &rb)
{
    if (EPI == EPI_SWIGLU) {
        ra = u, rb = u + a.m / 2;
    } else if (EPI == EPI_ROPE_KV) {
        // branch-free: the weight loads that follow must not sit under a condition (their count has to be static)
        const int hd2 = a.d >> 1, nqk = (a.h + a.g) * hd2;
        const int uq = min(u, nqk - 1), j = div_half_dim(uq, hd2), t = uq - j * hd2;
        const int rq = j * a.d + t, rv = (a.h + a.g) * a.d + 2 * (u - nqk);
        ra = u < nqk ? rq : rv;
        rb = u < nqk ? rq + hd2 : rv + 1;
    } else {
        ra = 2 * u, rb = min(2 * u + 1, a.m - 1);
    }
}

// what the epilogue of unit u reads besides the two sums, as raw bits: requested before the weight stream starts and
// not touched until the end (any use, even a conversion, would make the wavefront wait for it on the spot).  Every
// lane requests something valid -- no load under a condition, the count of requests in flight stays static.
template <int EPI>
__device__ __forceinline__ float2 epi_fetch(const GemvArgs &a, int i, const RowInfo &ri, int u)
{
    float2 pre = make_float2(0.0f, 0.0f);
    int ra, rb;
    unit_rows_r<EPI>(a, u, ra, rb);
    const size_t base = (size_t)i * a.m;
    if (EPI == EPI_RESID_F32) {
        const uint16_t *xr = (const uint16_t *)a.resid;
        pre = make_float2(__uint_as_float((uint32_t)xr[base + ra]), __uint_as_float((uint32_t)xr[base + rb]));
    } else if (EPI == EPI_RESID_F16) {
        const float *xr = (const float *)a.resid;
        pre = make_float2(xr[base + ra], xr[base + rb]);
    } else if (EPI == EPI_ROPE_KV) {
        const int hd2 = a.d >> 1, nqk = (a.h + a.g) * hd2;
        const int t = u < nqk ? u - div_half_dim(u, hd2) * hd2 : 0;
        pre = *(const float2 *)(a.rope + ((size_t)ri.pos * hd2 + t) * 2);                          // cos, sin
    }
    return pre;
}

template <int EPI>
__device__ __forceinline__ void epi_store(const GemvArgs &a, int i, const RowInfo &ri, int u, float va, float vb, float2 pre)
{
    int ra, rb;
    unit_rows_r<EPI>(a, u, ra, rb);
    const size_t base = (size_t)i * a.m;
    if (EPI == EPI_F16) {
        a.out_f16[base + ra] = f2h(va);
        if (2 * u + 1 < a.m) a.out_f16[base + rb] = f2h(vb);
    } else if (EPI == EPI_RESID_F32) {
        a.out_f32[base + ra] = h2f((uint16_t)__float_as_uint(pre.x)) + va;
        if (2 * u + 1 < a.m) a.out_f32[base + rb] = h2f((uint16_t)__float_as_uint(pre.y)) + vb;
    } else if (EPI == EPI_RESID_F16) {
        a.out_f16[base + ra] = f2h(pre.x + va);
        if (2 * u + 1 < a.m) a.out_f16[base + rb] = f2h(pre.y + vb);
    } else if (EPI == EPI_SWIGLU) {
        a.out_f16[(size_t)i * (a.m / 2) + u] = f2h(va / (1.0f + expf(-va)) * vb);
    } else {  // EPI_ROPE_KV
        const int hd2 = a.d >> 1, nqk = (a.h + a.g) * hd2;
        const size_t tok = ((size_t)ri.slot * a.kv_capacity + ri.pos) * (size_t)(a.g * a.d);
        if (u < nqk) {
            const int j = div_half_dim(u, hd2), t = u - j * hd2;
            const float oa = va * pre.x - vb * pre.y, ob = va * pre.y + vb * pre.x;
            uint16_t *dst = (j < a.h) ? a.out_f16 + (size_t)i * (a.h * a.d) + (size_t)j * a.d + t
                                      : a.kcache + tok + (size_t)(j - a.h) * a.d + t;
            dst[0] = f2h(oa), dst[hd2] = f2h(ob);
        } else {
            uint16_t *dst = a.vcache + tok + 2 * (size_t)(u - nqk);
            dst[0] = f2h(va), dst[1] = f2h(vb);
        }
    }
}

constexpr int kRSlots = 2;                // slots in flight (the schedule of the stream is written for two)

// Rows per slot, R.  Small slots shorten what is left to compute after the last byte has arrived and let the
// arithmetic follow the stream more closely; large ones keep more bytes in flight.  Measured on the 7B layer: two rows
// for rows of up to 4096 columns (four rows: +3 us per layer; one row: +2.7 us), except when a wavefront owns four
// rows or fewer (the output projection: one row per slot is 0.6 us faster); one row for rows beyond 4096 columns, whose
// lanes keep 64 to 96 registers of x: with two rows the six-chunk variant needed 382 registers (+1.5 us), and the four-chunk
// variant spilled to scratch memory (57344 x 8192 at one row: 166 us against 43.5 us with one row per slot).
template <int NG>
constexpr int rows_per_slot(bool few_rows)
{
    return NG >= 4 ? 1 : (few_rows ? 1 : 2);
}
template <int NG>
constexpr int kMaxRowsPerSlot = NG >= 4 ? 1 : 2;          // what the launcher instantiates

// grid: x = workgroups (at most one per CU and pass), y = pass: NR rows of x that share one pass over the weights (a
// batch of two to four decode rows: the stream is the same, the dot products of a group are taken once per row on the
// words decoded once; a ragged last pass re-reads the last row and stores nothing for it)
// DEV: the position of the (single) row comes from the device-resident descriptor a.seqs.dev instead of a.pos0 / a.slot0
// (a captured launch is then valid for later positions too); only the two variants that need a position have it.
// Several rows per pass keep NR times the x registers: those variants are compiled for one wavefront per SIMD (which is
// how every variant runs: one workgroup per CU), so that the allocator may use the whole register file instead of spilling.
// FP16W: the matrix is plain fp16, a.wh [m,k] (the fp16 models of Sec. 5.1): the same stream with four 16-byte loads per lane,
// row and chunk instead of one load and a scale -- load j of chunk c brings columns 2048 c + 512 j + 8 lane .. + 7, a contiguous
// kilobyte per instruction -- and nothing to decode: x is staged in plain column order and a load meets its eight x values
// in four v_dot2_f32_f16.  Columns past the end of a row meet x = 0 (the staging zero-fills), so no lane is masked.
// Q3W: the matrix is 3-bit in the GPU-native word layout (Sec. 5.3; gemv_q3.hip describes it): twelve bytes and one scale per
// lane, row and chunk, x staged in plain column order under the group mapping of the 4-bit stream, the decode of a group
// (24 vector operations into 16 ready fp16 pairs of three scale classes) ahead of its 16 dot products.
template <int XMODE, int EPI, int NG, int R, bool DEV = false, int NR = 1, int WM = W_Q4>
__global__ __launch_bounds__(kRThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemv_q4_reg_kernel(GemvArgs a)
{
    static_assert(NR == 1 || (XMODE != X_ATTN_MERGE && !DEV), "several rows per pass: plain and normalising prologues, host descriptor");
    constexpr bool FP16W = WM == W_F16, Q3W = WM == W_Q3;
    static_assert(WM == W_Q4 || NR == 1, "fp16 and 3-bit weights: one row of x per pass");
    constexpr int LW = FP16W ? 4 : 1;                              // 16-byte loads per lane, row and chunk
    constexpr int NSLOT = kRSlots, E = R * NG;
    constexpr int kResPitch = NR * (kRMaxUnits * 2 + 4);
    constexpr int kFirstRagged = NG >= 4 ? NG - 2 : NG - 1;        // first chunk of 2048 columns that a row may end in
    __shared__ __align__(16) uint16_t xs[NR * NG * 2048];
    __shared__ float red[NR * kRWaves];
    __shared__ float res_all[kRWaves][kResPitch];              // one sum per matrix row of the wavefront and row of x (+ the dead rows of a last slot)
    // The arguments this variant uses, in scalar registers from here on: one round of scalar loads and one wait ahead of
    // the first request, none at the place of a first use further down (where the stream or the epilogue would wait).
    if (FP16W) asm volatile("" ::"s"(a.x), "s"(a.wh), "s"(a.m), "s"(a.k), "s"(a.units_div), "s"(a.units_mod));
    else asm volatile("" ::"s"(a.x), "s"(a.q), "s"(a.s), "s"(a.m), "s"(a.k), "s"(a.gshift), "s"(a.units_div), "s"(a.units_mod));
    if (XMODE == X_F16_NORM || XMODE == X_F32_NORM) asm volatile("" ::"s"(a.norm_w), "s"(a.eps));
    if (XMODE == X_ATTN_MERGE) asm volatile("" ::"s"(a.part), "s"(a.part_splits), "s"(a.part_stride), "s"(a.part_used), "s"(a.h), "s"(a.d));
    if (EPI == EPI_RESID_F32) asm volatile("" ::"s"(a.out_f32), "s"(a.resid));
    if (EPI == EPI_RESID_F16) asm volatile("" ::"s"(a.out_f16), "s"(a.resid));
    if (EPI == EPI_F16 || EPI == EPI_SWIGLU) asm volatile("" ::"s"(a.out_f16));
    if (EPI == EPI_ROPE_KV) asm volatile("" ::"s"(a.out_f16), "s"(a.rope), "s"(a.h), "s"(a.g), "s"(a.d), "s"(a.pos0), "s"(a.slot0));
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i0 = blockIdx.y * NR;
    const int i = i0;                                          // NR == 1: the row
    int irow[NR];                                              // a ragged last pass re-reads the last row (never stored)
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) irow[xr] = min(i0 + xr, a.n - 1);
    const int k = a.k, G = k >> 5, kw = k >> 3, SG = scales_per_row(k, a.gshift);
    const int U = unit_count_r<EPI>(a);
    const int W = gridDim.x * kRWaves, wg = blockIdx.x * kRWaves + wave;
    const int mine = a.units_div + (wg < a.units_mod ? 1 : 0); // units wg, wg + W, .. below U, the division done by the host; <= kRMaxUnits
    float *res = res_all[wave];

    // ---- what the epilogue reads, then the x row, then the first slots: requested in the order they are needed ----
    int rpos[NR], rslot[NR];                                   // position and cache slot of every row (rotary + append epilogue)
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) {
        rpos[xr] = rslot[xr] = 0;
        if (EPI == EPI_ROPE_KV) {
            if (!DEV && a.n == 1) {
                rpos[xr] = a.pos0, rslot[xr] = a.slot0;            // the host resolved the only row: no table walk up front
            } else {
                const RowInfo t = row_info(a.seqs, irow[xr]);      // DEV: scalar loads of the descriptor
                rpos[xr] = t.pos, rslot[xr] = t.slot;
            }
        }
    }

    // pass p of the staging covers chunk p of 2048 columns: thread t holds word t & 3 of group 64 p + (t >> 2)
    constexpr bool kNorm = (XMODE == X_F16_NORM || XMODE == X_F32_NORM), kMerge = (XMODE == X_ATTN_MERGE);
    constexpr int MS = kAttnMergeSplits;
    u32x4_t xraw[NR][NG], xraw2[NR][XMODE == X_F32_NORM ? NG : 1], wnr[kNorm ? NG : 1];
    // X_ATTN_MERGE: x is the attention output, still in split form.  The thread's 8 elements belong to one head; it
    // reads their accumulators and the (max, sum) pair of every split (splits past the used ones re-read the last)
    u32x4_t pacc[kMerge ? NG : 1][kMerge ? MS : 1];            // 8 normalised outputs of the split, fp16
    float2 pml[kMerge ? NG : 1][kMerge ? MS : 1];
    int used = 0;                                              // splits that hold tokens: ceil((pos + 1) / chunk)
    if (kMerge && DEV) {
        const int pos = row_info(a.seqs, 0).pos;
        used = attn_fold_used(pos, attn_fold_chunk(pos + 1, a.part_splits));
    } else if (kMerge) {
        used = a.part_used;                                        // the host knew the position: no division up front
    }
    auto x_loads = [&]() {
#pragma unroll
    for (int p = 0; p < NG; ++p) {
        const int c8 = min(p * kRThreads + tid, kw - 1);
        if (kMerge) {
            const int head = (c8 * 8) / a.d, e = c8 * 8 - head * a.d;
            const float *pb = a.part + ((size_t)i * a.h + head) * (size_t)a.part_splits * a.part_stride;
#pragma unroll
            for (int s = 0; s < MS; ++s) {
                const float *ps = pb + (size_t)min(s, used - 1) * a.part_stride;
                pacc[p][s] = *(const u32x4_t *)((const uint16_t *)ps + e);
                pml[p][s] = *(const float2 *)(ps + (a.d >> 1));
            }
        } else if (XMODE == X_F32_NORM) {
#pragma unroll
            for (int xr = 0; xr < NR; ++xr) {
                xraw[xr][p] = *(const u32x4_t *)((const float *)a.x + (size_t)irow[xr] * k + (size_t)c8 * 8);
                xraw2[xr][p] = *(const u32x4_t *)((const float *)a.x + (size_t)irow[xr] * k + (size_t)c8 * 8 + 4);
            }
        } else {
#pragma unroll
            for (int xr = 0; xr < NR; ++xr) xraw[xr][p] = *(const u32x4_t *)((const uint16_t *)a.x + (size_t)irow[xr] * k + (size_t)c8 * 8);
        }
        if (kNorm) wnr[p] = *(const u32x4_t *)(a.norm_w + (size_t)c8 * 8);
    }
    };
    // The x row goes out ahead of the weights: it is needed first and is small.  That holds for the partials of
    // X_ATTN_MERGE too, although they are 24 requests per thread: returns are counted in order, so behind the slots the
    // merge arithmetic could only start once the weights were there; ahead of them it runs while they are on their way
    // (0.4 us per call at the 7B shape).
    x_loads();

    struct Slot {
        u32x4_t w[E * LW];
        uint16_t sc[FP16W ? 1 : E];
    };
    // entry e = rr * NG + c: row rr of the slot (unit j0 + rr / 2, its first or second row), chunk c
    // The requests of a slot stay together in program order (scheduling barriers on both sides): the wait before a
    // consume is a count of younger requests, and one request of this slot issued late would make it cover the
    // other slot as well.
    // The rows of a wavefront in sequence: row t is row t & 1 of its unit t >> 1; slot si holds rows si R .. si R + R - 1.
    auto slot_load = [&](Slot &s, int si) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            // units past the end re-read the unit before them -- the other half of the same slot, still on its way or
            // in the L2, and a different address per wavefront (one shared address would queue every wavefront of
            // the grid on the same few cache lines) -- and are dropped
            const int t = si * R + rr, j = t >> 1;
            const int uj = wg + j * W, ub = wg + max(j - 1, 0) * W;
            const int u = uj < U ? uj : (ub < U ? ub : min(wg, U - 1));
            int rows[2];
            unit_rows_r<EPI>(a, u, rows[0], rows[1]);
            const int row = __builtin_amdgcn_readfirstlane((t & 1) ? rows[1] : rows[0]);     // uniform: row bases in scalar registers
            if constexpr (FP16W) {
                const uint16_t *wrow = a.wh + (size_t)row * k;
#pragma unroll
                for (int c = 0; c < NG; ++c)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int pk = c * 256 + j * 64 + lane;    // 16-byte packet of the row; past the end: the last one (it meets x = 0)
                        const int pc = (c >= kFirstRagged) ? min(pk, kw - 1) : pk;
                        s.w[(rr * NG + c) * 4 + j] = stream_load((const u32x4_t *)(wrow + (size_t)pc * 8));
                    }
            } else if constexpr (Q3W) {
                const uint32_t *qrow = a.q + (size_t)row * G * 3;
                const uint16_t *srow = a.s + (size_t)row * G;
#pragma unroll
                for (int c = 0; c < NG; ++c) {
                    const int gi = (c >= kFirstRagged) ? min(c * 64 + lane, G - 1) : c * 64 + lane;
                    const uint32_t *p3 = qrow + gi * 3;              // consecutive lanes read consecutive 12-byte groups
                    u32x4_t w3 = {0u, 0u, 0u, 0u};
                    w3.x = stream_load(p3), w3.y = stream_load(p3 + 1), w3.z = stream_load(p3 + 2);
                    s.w[rr * NG + c] = w3;
                    s.sc[rr * NG + c] = srow[gi];
                }
            } else {
            const uint32_t *qrow = a.q + (size_t)row * kw;
            const uint16_t *srow = a.s + (size_t)row * SG;
#pragma unroll
            for (int c = 0; c < NG; ++c) {
                // chunks that can reach past the row (NG = 4, 6 also serve rows one chunk shorter) are clamped
                const int gi = (c >= kFirstRagged) ? min(c * 64 + lane, G - 1) : c * 64 + lane;
                s.w[rr * NG + c] = stream_load((const u32x4_t *)(qrow + gi * 4));
                s.sc[rr * NG + c] = srow[gi >> a.gshift];     // 1, 2 or 4 neighbouring lanes read the same scale
            }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    Slot sl[NSLOT];
#pragma unroll
    for (int t = 0; t < NSLOT; ++t) slot_load(sl[t], t);
    // behind the first slots in program order: its address arithmetic runs while they are in flight
    float2 pre[NR];
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) pre[xr] = epi_fetch<EPI>(a, irow[xr], RowInfo{0, rpos[xr], rslot[xr]}, lane < mine ? wg + lane * W : min(wg, U - 1));
    __builtin_amdgcn_sched_barrier(0);

    // ---- stage the (optionally RMS-normalised) x row in LDS as fp16, packet order [x0 x4 x1 x5 x2 x6 x3 x7] ----
    const float inv_k = 1.0f / (float)k;                           // ahead of the reduction it is used with
    float inv[NR];
    float xf[NR][kNorm ? NG : 1][8];
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) inv[xr] = 1.0f;
    if (kNorm) {
#pragma unroll
        for (int xr = 0; xr < NR; ++xr) {
            float ss = 0.0f;
#pragma unroll
            for (int p = 0; p < NG; ++p) {
                const bool on = (p * kRThreads + tid) < kw;
                if (XMODE == X_F32_NORM) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) xf[xr][p][e] = __uint_as_float(xraw[xr][p][e]), xf[xr][p][4 + e] = __uint_as_float(xraw2[xr][p][e]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        xf[xr][p][2 * e] = h2f((uint16_t)(xraw[xr][p][e] & 0xFFFFu)), xf[xr][p][2 * e + 1] = h2f((uint16_t)(xraw[xr][p][e] >> 16));
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    xf[xr][p][e] = on ? xf[xr][p][e] : 0.0f;
                    ss += xf[xr][p][e] * xf[xr][p][e];
                }
            }
            ss = wave_sum(ss);
            if (lane == 0) red[xr * kRWaves + wave] = ss;
        }
        wg_barrier();
#pragma unroll
        for (int xr = 0; xr < NR; ++xr) {
            float tot = 0.0f;
#pragma unroll
            for (int w = 0; w < kRWaves; ++w) tot += red[xr * kRWaves + w];
            inv[xr] = rms_scale(tot, inv_k, a.eps);
        }
    }
#pragma unroll
    for (int xr = 0; xr < NR; ++xr)
#pragma unroll
    for (int p = 0; p < NG; ++p) {
        u32x4_t o;
        if (kNorm) {
            uint16_t y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t ww = wnr[p][e >> 1];
                y[e] = f2h(xf[xr][p][e] * inv[xr] * h2f((uint16_t)((e & 1) ? (ww >> 16) : (ww & 0xFFFFu))));
            }
            if (WM != W_Q4) {
                o.x = (uint32_t)y[0] | ((uint32_t)y[1] << 16), o.y = (uint32_t)y[2] | ((uint32_t)y[3] << 16);
                o.z = (uint32_t)y[4] | ((uint32_t)y[5] << 16), o.w = (uint32_t)y[6] | ((uint32_t)y[7] << 16);
            } else {
                o.x = (uint32_t)y[0] | ((uint32_t)y[4] << 16), o.y = (uint32_t)y[1] | ((uint32_t)y[5] << 16);
                o.z = (uint32_t)y[2] | ((uint32_t)y[6] << 16), o.w = (uint32_t)y[3] | ((uint32_t)y[7] << 16);
            }
        } else if (kMerge) {
            // out = sum_s acc_s e^(m_s - M) / sum_s l_s e^(m_s - M), rounded to fp16 like the stand-alone merge
            const bool on = (p * kRThreads + tid) < kw;
            float mm = -INFINITY;
#pragma unroll
            for (int s = 0; s < MS; ++s) mm = (s < used) ? fmaxf(mm, pml[p][s].x) : mm;
            float num[8], den = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) num[e] = 0.0f;
#pragma unroll
            for (int s = 0; s < MS; ++s) {
                // the split kernel left out_s = acc_s / l_s (fp16) and (m_s, l_s): weight of the split = l_s e^(m_s - M)
                const float w = (s < used) ? __expf(pml[p][s].x - mm) * pml[p][s].y : 0.0f;
                den += w;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t ow = pacc[p][s][j];
                    num[2 * j] += w * h2f((uint16_t)(ow & 0xFFFFu)), num[2 * j + 1] += w * h2f((uint16_t)(ow >> 16));
                }
            }
            // one division per head instead of one per element (a dozen instructions each, ahead of the whole stream);
            // den > 0: the first split holds a token
            const float rden = on ? 1.0f / den : 0.0f;
            uint16_t y[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = f2h(num[e] * rden);
            if (WM != W_Q4) {
                o.x = (uint32_t)y[0] | ((uint32_t)y[1] << 16), o.y = (uint32_t)y[2] | ((uint32_t)y[3] << 16);
                o.z = (uint32_t)y[4] | ((uint32_t)y[5] << 16), o.w = (uint32_t)y[6] | ((uint32_t)y[7] << 16);
            } else {
                o.x = (uint32_t)y[0] | ((uint32_t)y[4] << 16), o.y = (uint32_t)y[1] | ((uint32_t)y[5] << 16);
                o.z = (uint32_t)y[2] | ((uint32_t)y[6] << 16), o.w = (uint32_t)y[3] | ((uint32_t)y[7] << 16);
            }
        } else {
            const bool on = (p * kRThreads + tid) < kw;
            const u32x4_t r = xraw[xr][p];
            if (WM != W_Q4) {
                o = r;
            } else {
                o.x = __builtin_amdgcn_perm(r.z, r.x, 0x05040100u), o.y = __builtin_amdgcn_perm(r.z, r.x, 0x07060302u);
                o.z = __builtin_amdgcn_perm(r.w, r.y, 0x05040100u), o.w = __builtin_amdgcn_perm(r.w, r.y, 0x07060302u);
            }
            if (!on) o = u32x4_t{0u, 0u, 0u, 0u};
        }
        // the thread holds columns 2048 p + 8 tid .. + 7: word tid & 3 of group 64 p + (tid >> 2), or (fp16 weights) the packet that
        // load tid >> 6 of lane tid & 63 meets
        if (FP16W) *(u32x4_t *)(xs + xr * (NG * 2048) + (((p * 4 + (tid >> 6)) << 6) + (tid & 63)) * 8) = o;
        else *(u32x4_t *)(xs + xr * (NG * 2048) + (((p * 4 + (tid & 3)) << 6) + (tid >> 2)) * 8) = o;
    }
    wg_barrier();
    // the lane's share of x: group c * 64 + lane of every chunk, and the offset term of each group
    u32x4_t xv[NR][NG][4];
    float cr[NR][NG];
#pragma unroll
    for (int xr = 0; xr < NR; ++xr)
#pragma unroll
    for (int c = 0; c < NG; ++c) {
        float sa = 0.0f, sb = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            xv[xr][c][j] = *(const u32x4_t *)(xs + xr * (NG * 2048) + (((c * 4 + j) << 6) + lane) * 8);
            sa = dot2(xv[xr][c][j].x, 0x3C003C00u, sa), sb = dot2(xv[xr][c][j].y, 0x3C003C00u, sb);
            sa = dot2(xv[xr][c][j].z, 0x3C003C00u, sa), sb = dot2(xv[xr][c][j].w, 0x3C003C00u, sb);
        }
        cr[xr][c] = FP16W ? 0.0f : 1032.0f * sa + 72.0f * sb;
        if constexpr (Q3W) {                                       // pair p = 4 j + word of the packet; its scale class as in the decode
            float sc3[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                sc3[q3n_class(4 * j)] = dot2(0x3C003C00u, xv[xr][c][j].x, sc3[q3n_class(4 * j)]);
                sc3[q3n_class(4 * j + 1)] = dot2(0x3C003C00u, xv[xr][c][j].y, sc3[q3n_class(4 * j + 1)]);
                sc3[q3n_class(4 * j + 2)] = dot2(0x3C003C00u, xv[xr][c][j].z, sc3[q3n_class(4 * j + 2)]);
                sc3[q3n_class(4 * j + 3)] = dot2(0x3C003C00u, xv[xr][c][j].w, sc3[q3n_class(4 * j + 3)]);
            }
            cr[xr][c] = 1028.0f * sc3[0] + 132.0f * sc3[1] + 20.0f * sc3[2];
        }
    }
    bool chunk_on[NG];                                             // lanes past the last group of the row contribute nothing
#pragma unroll
    for (int c = 0; c < NG; ++c) chunk_on[c] = c * 64 + lane < G;

    // ---- the stream ------------------------------------------------------------------------------------------
    auto consume = [&](const Slot &s, int j0) {
        float acc[R * NR];                                         // value rr * NR + xr: row rr of the slot, row xr of x
#pragma unroll
        for (int v = 0; v < R * NR; ++v) acc[v] = 0.0f;
        // in the order the requests went out (row by row): every group is used as soon as it has arrived
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int c = 0; c < NG; ++c) {
                if constexpr (FP16W) {
                    float dsum = 0.0f;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const u32x4_t wv = s.w[(rr * NG + c) * 4 + j];
                        dsum = dot2(wv.x, xv[0][c][j].x, dsum), dsum = dot2(wv.y, xv[0][c][j].y, dsum);
                        dsum = dot2(wv.z, xv[0][c][j].z, dsum), dsum = dot2(wv.w, xv[0][c][j].w, dsum);
                    }
                    acc[rr] += dsum;
                    continue;
                }
                float scv = h2f(s.sc[FP16W ? 0 : rr * NG + c]);
                if (c >= kFirstRagged) scv = chunk_on[c] ? scv : 0.0f;
                if constexpr (Q3W) {
                    uint32_t pk[16];
                    const u32x4_t w3 = s.w[rr * NG + c];
                    q3n_decode(w3.x, w3.y, w3.z, pk);
                    float a3[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        a3[q3n_class(4 * j)] = dot2(pk[4 * j], xv[0][c][j].x, a3[q3n_class(4 * j)]);
                        a3[q3n_class(4 * j + 1)] = dot2(pk[4 * j + 1], xv[0][c][j].y, a3[q3n_class(4 * j + 1)]);
                        a3[q3n_class(4 * j + 2)] = dot2(pk[4 * j + 2], xv[0][c][j].z, a3[q3n_class(4 * j + 2)]);
                        a3[q3n_class(4 * j + 3)] = dot2(pk[4 * j + 3], xv[0][c][j].w, a3[q3n_class(4 * j + 3)]);
                    }
                    acc[rr] += scv * (a3[0] + a3[1] * 0.125f + a3[2] * 0.015625f - cr[0][c]);
                    continue;
                }
                if constexpr (NR == 1) {
                    acc[rr] += scv * group_dot_r(s.w[rr * NG + c], xv[0][c], cr[0][c]);
                } else {
                    // the sixteen decoded pairs of the group once, a dot product per row of x
                    const u32x4_t wq = s.w[rr * NG + c];
                    uint32_t dq[16];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint32_t w = wq[j], w8 = w >> 8;
                        dq[4 * j] = and_or(w, 0x000F000Fu, 0x64006400u), dq[4 * j + 1] = and_or(w, 0x00F000F0u, 0x64006400u);
                        dq[4 * j + 2] = and_or(w8, 0x000F000Fu, 0x64006400u), dq[4 * j + 3] = and_or(w8, 0x00F000F0u, 0x64006400u);
                    }
#pragma unroll
                    for (int xr = 0; xr < NR; ++xr) {
                        float accA = 0.0f, accB = 0.0f;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            accA = dot2(dq[4 * j], xv[xr][c][j].x, accA), accB = dot2(dq[4 * j + 1], xv[xr][c][j].y, accB);
                            accA = dot2(dq[4 * j + 2], xv[xr][c][j].z, accA), accB = dot2(dq[4 * j + 3], xv[xr][c][j].w, accB);
                        }
                        acc[rr * NR + xr] += scv * (accA + accB * 0.0625f - cr[xr][c]);
                    }
                }
            }
        // res[t * NR + xr] = sum of the wavefront's row t against row xr of x
        static_assert(R == 1 || R == 2, "slots of one or two rows");
        if constexpr (NR > 1) {
            const float r = reduce_many<R * NR>(acc, lane);            // lane l: the total of value l % (R NR)
            if (lane < R * NR) res[j0 * (R * NR) + lane] = r;
        } else if (R == 2) {
            const float r = reduce2(acc[0], acc[R > 1 ? 1 : 0], lane);
            if (lane < 2) res[j0 * 2 + lane] = r;
        } else {
            const float r = reduce1(acc[0]);
            if (lane == 0) res[j0] = r;
        }
    };
    // Slots of the wavefront: ns of them, NSLOT in flight.  Every path below is straight-line in its loads -- none
    // sits under a condition that merges back -- so the wait before a consume counts exactly the loads requested after
    // its slot, and nothing is requested past the end (a wavefront does not retire before its loads have returned).
    // Steady state: a step consumes a slot and refills it, NSLOT steps per trip.  What is left after the last full
    // trip, NSLOT + extra slots, runs through the variant of the tail written for that `extra`: `extra` more steps
    // with a refill, then one consume for every slot still in flight, in order.
    const int ns = (2 * mine + R - 1) / R;
    int s = 0;
#pragma unroll 1
    for (; s + 2 * NSLOT <= ns; s += NSLOT) {                      // refills up to slot s + 2 NSLOT - 1 exist
#pragma unroll
        for (int t = 0; t < NSLOT; ++t) {
            consume(sl[t], s + t);
            slot_load(sl[t], s + t + NSLOT);
        }
    }
    auto tail = [&](auto extra_c) {
        constexpr int EXTRA = decltype(extra_c)::value;
#pragma unroll
        for (int t = 0; t < EXTRA; ++t) {
            consume(sl[t], s + t);
            slot_load(sl[t], s + t + NSLOT);
        }
#pragma unroll
        for (int t = EXTRA; t < NSLOT; ++t) consume(sl[t], s + t);
#pragma unroll
        for (int t = 0; t < EXTRA; ++t) consume(sl[t], s + t + NSLOT);
    };
    const int left = ns - s;                                       // 0 .. 2 NSLOT - 1
    if (left >= NSLOT) {
        const int extra = left - NSLOT;
        if (extra == 0) tail(std::integral_constant<int, 0>{});
        else if (extra == 1) tail(std::integral_constant<int, 1>{});
        else if (NSLOT > 2 && extra == 2) tail(std::integral_constant<int, (NSLOT > 2 ? 2 : 0)>{});
        else if (NSLOT > 3) tail(std::integral_constant<int, (NSLOT > 3 ? 3 : 0)>{});
    } else {
        // fewer slots than are in flight (tiny matrices): the slots past the end hold re-read rows and are skipped
#pragma unroll
        for (int t = 0; t < NSLOT - 1; ++t)
            if (t < left) consume(sl[t], t);
    }

    // ---- epilogue: lane jj finishes the wavefront's unit jj ----------------------------------------------------
    if (lane < mine) {
#pragma unroll
        for (int xr = 0; xr < NR; ++xr)
            if (i0 + xr < a.n)
                epi_store<EPI>(a, i0 + xr, RowInfo{0, rpos[xr], rslot[xr]}, wg + lane * W, res[(lane * 2) * NR + xr], res[(lane * 2 + 1) * NR + xr], pre[xr]);
    }
}

template <int XMODE, int EPI, int NG, int WM = W_Q4>
hipError_t launch_ng(const GemvArgs &a_in, hipStream_t stream)
{
    GemvArgs a = a_in;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
        cus = v;                                                   // one workgroup per CU (two per CU measured 1 us per layer slower)
    }
    const int U = (EPI == EPI_SWIGLU || EPI == EPI_ROPE_KV) ? a.m / 2 : (a.m + 1) / 2;
    // rows of x that share a pass over the weights: four where a lane's x is 32 registers per row (k <= 4096), two up to
    // k = 8192, one beyond (the variants that would not fit 256 vector registers are not built)
    const int nr = (WM != W_Q4 || XMODE == X_ATTN_MERGE || a.n < 2 || NG > 4) ? 1 : (a.n >= 3 && NG <= 2 ? 4 : 2);
    const int passes = (a.n + nr - 1) / nr;
    // one workgroup per CU, shared between the passes; never fewer than what keeps a wavefront within kRMaxUnits
    int gx = std::max(1, cus / std::min(passes, 8));
    gx = std::min(gx, (U + kRWaves - 1) / kRWaves);
    gx = std::max(gx, (U + kRWaves * kRMaxUnits - 1) / (kRWaves * kRMaxUnits));
    const bool few_rows = 2 * ((U + gx * kRWaves - 1) / (gx * kRWaves)) <= 4;      // rows a wavefront owns
    constexpr bool kHasPos = EPI == EPI_ROPE_KV || XMODE == X_ATTN_MERGE;
    // (the merge prologue keeps the split accumulators of the row in registers until x is staged: one-row slots beside them --
    // 5120 x 5120 with the merge folded in 0.7 us faster than with two-row slots)
    const bool one = rows_per_slot<NG>(few_rows) == 1 || XMODE == X_ATTN_MERGE;
    a.units_div = U / (gx * kRWaves), a.units_mod = U % (gx * kRWaves);
    const dim3 grid(gx, passes);
    if constexpr (WM == W_F16) {                                   // a row is four times the bytes: one row per slot throughout
        if constexpr (kHasPos) {
            if (a.n == 1 && a.pos0 < 0) {
                if (a.seqs.dev == nullptr) return hipErrorInvalidValue;
                hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, true, 1, W_F16>), grid, dim3(kRThreads), 0, stream, a);
                return hipGetLastError();
            }
        }
        hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, false, 1, W_F16>), grid, dim3(kRThreads), 0, stream, a);
        return hipGetLastError();
    }
    if constexpr (WM == W_Q3) {                                    // rows per slot as on the 4-bit stream
        if constexpr (kHasPos) {
            if (a.n == 1 && a.pos0 < 0) {
                if (a.seqs.dev == nullptr) return hipErrorInvalidValue;
                if (one) hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, true, 1, W_Q3>), grid, dim3(kRThreads), 0, stream, a);
                else hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, kMaxRowsPerSlot<NG>, true, 1, W_Q3>), grid, dim3(kRThreads), 0, stream, a);
                return hipGetLastError();
            }
        }
        if (one) hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, false, 1, W_Q3>), grid, dim3(kRThreads), 0, stream, a);
        else hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, kMaxRowsPerSlot<NG>, false, 1, W_Q3>), grid, dim3(kRThreads), 0, stream, a);
        return hipGetLastError();
    }
    if constexpr (kHasPos) {
        if (a.n == 1 && a.pos0 < 0) {                              // position from the device-resident descriptor
            if (a.seqs.dev == nullptr) return hipErrorInvalidValue;
            if (one) hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, true>), grid, dim3(kRThreads), 0, stream, a);
            else hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, kMaxRowsPerSlot<NG>, true>), grid, dim3(kRThreads), 0, stream, a);
            return hipGetLastError();
        }
    }
    if constexpr (XMODE != X_ATTN_MERGE && NG <= 2) {
        if (nr == 4) {                                             // one-row slots: 8 sums per slot would not fit
            hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, false, 4>), grid, dim3(kRThreads), 0, stream, a);
            return hipGetLastError();
        }
        if (nr == 2) {
            if (one) hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, false, 2>), grid, dim3(kRThreads), 0, stream, a);
            else hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, kMaxRowsPerSlot<NG>, false, 2>), grid, dim3(kRThreads), 0, stream, a);
            return hipGetLastError();
        }
    }
    if constexpr (XMODE != X_ATTN_MERGE && (NG == 3 || NG == 4)) {
        if (nr == 2) {
            hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1, false, 2>), grid, dim3(kRThreads), 0, stream, a);
            return hipGetLastError();
        }
    }
    if (one) hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, 1>), grid, dim3(kRThreads), 0, stream, a);
    else hipLaunchKernelGGL((gemv_q4_reg_kernel<XMODE, EPI, NG, kMaxRowsPerSlot<NG>>), grid, dim3(kRThreads), 0, stream, a);
    return hipGetLastError();
}

template <int XMODE, int EPI, int WM = W_Q4>
hipError_t launch_xe(const GemvArgs &a, hipStream_t stream)
{
    const int ng = (a.k + 2047) / 2048;
    if (ng <= 1) return launch_ng<XMODE, EPI, 1, WM>(a, stream);
    if (ng == 2) return launch_ng<XMODE, EPI, 2, WM>(a, stream);
    if (ng == 3) return launch_ng<XMODE, EPI, 3, WM>(a, stream);     // hidden 5120: no dead fourth chunk
    if (ng <= 4) return launch_ng<XMODE, EPI, 4, WM>(a, stream);
    return launch_ng<XMODE, EPI, 6, WM>(a, stream);
}

}  // namespace

}  // namespace relax
