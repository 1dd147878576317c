// Matrix-vector kernel for rows longer than the x registers of one wavefront hold (12288 < k <= 32768: the down projection
// of the 70B and 13B layer shapes at one row; Relax, Sec. 4.2 decode_q4 case study, Sec. 5.1 batch-1 decoding).
//
// The stream of gemv_reg_kernel.h with the row split over the four wavefronts of a workgroup instead of walked by one:
// chunk c of wavefront w is columns 2048 (4 c + w) .. + 2047 of every row of the workgroup, so a lane keeps at most
// 4 x 16 registers of x, a slot is one row or a row pair (R NG 16-byte loads and scales per lane: 32 KB per workgroup in
// flight with two slots), and the four partial sums of a row meet in LDS after the stream has drained.  x needs no staging: a lane reads the 64 bytes of each of
// its groups straight from global memory (x is a few tens of KB and stays in the L2), which only the plain prologue allows;
// the epilogues are those of a row pair (plain, fp16 and fp32 residual), their inputs fetched ahead of the stream.
// With a quarter of a row per wavefront a lane has room for several rows of x: NR rows (a few decode rows) share one pass
// over the weights, the words of a group decoded once and met by every row -- which is why rows of 8193..12288 columns come
// here from two rows of x on, where the one-wavefront-per-row kernel would stream the matrix once per row.
#include "gemv_reg_kernel.h"

namespace relax {

namespace {

constexpr int kLongMaxUnits = 64;         // row pairs per workgroup: thread j of the first wavefront finishes pair j

template <int EPI, int NG, int R, int NR>
__global__ __launch_bounds__(kRThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemv_q4_long_kernel(GemvArgs a)
{
    static_assert(EPI == EPI_F16 || EPI == EPI_RESID_F16 || EPI == EPI_RESID_F32, "row-pair epilogues");
    __shared__ float part[kRWaves][(2 * kLongMaxUnits + 2) * NR];   // [wavefront][row of the workgroup][row of x]
    asm volatile("" ::"s"(a.x), "s"(a.q), "s"(a.s), "s"(a.m), "s"(a.k), "s"(a.gshift), "s"(a.units_div), "s"(a.units_mod));
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i0 = blockIdx.y * NR;                                // first row of x of the pass; a ragged last pass re-reads the last row
    int irow[NR];
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) irow[xr] = min(i0 + xr, a.n - 1);
    const int k = a.k, G = k >> 5, kw = k >> 3, SG = scales_per_row(k, a.gshift);
    const int U = unit_count_r<EPI>(a);
    const int W = gridDim.x, wg = blockIdx.x;
    const int mine = a.units_div + (wg < a.units_mod ? 1 : 0);     // pairs wg, wg + W, ..; <= kLongMaxUnits

    // what the epilogue reads, then the first two rows of the stream, then x
    float2 pre[NR];
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) pre[xr] = epi_fetch<EPI>(a, irow[xr], RowInfo{0, 0, 0}, tid < mine ? wg + tid * W : min(wg, U - 1));
    int gi[NG];
    bool on[NG];
#pragma unroll
    for (int c = 0; c < NG; ++c) {
        const int g = (4 * c + wave) * 64 + lane;                  // the lane's group of the chunk; past the end: the last group, scale 0
        on[c] = g < G;
        gi[c] = min(g, G - 1);
    }
    static_assert(R == 1 || R == 2, "a slot is a row or a row pair");
    struct Slot {
        u32x4_t w[R * NG];
        uint16_t sc[R * NG];
    };
    // R = 1: slot t = row t & 1 of pair wg + (t >> 1) W; R = 2: slot t = pair wg + t W; past the end: the last row again
    auto slot_load = [&](Slot &s, int t) {
        __builtin_amdgcn_sched_barrier(0);
        const int u = min(wg + (R == 2 ? t : t >> 1) * W, U - 1);
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int row = min(2 * u + (R == 2 ? rr : (t & 1)), a.m - 1);
            const uint32_t *qrow = a.q + (size_t)row * kw;
            const uint16_t *srow = a.s + (size_t)row * SG;
#pragma unroll
            for (int c = 0; c < NG; ++c) {
                s.w[rr * NG + c] = stream_load((const u32x4_t *)(qrow + gi[c] * 4));
                s.sc[rr * NG + c] = srow[gi[c] >> a.gshift];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    Slot sl[2];
    slot_load(sl[0], 0);
    slot_load(sl[1], 1);

    // x of the lane's groups in the word order of the decode: [x0 x4 | x1 x5 | x2 x6 | x3 x7] per 8-column packet
    u32x4_t xv[NR][NG][4];
    float cr[NR][NG];
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) {
        const uint16_t *xrow = (const uint16_t *)a.x + (size_t)irow[xr] * k;
#pragma unroll
        for (int c = 0; c < NG; ++c) {
            float sa = 0.0f, sb = 0.0f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const u32x4_t r = *(const u32x4_t *)(xrow + (size_t)gi[c] * 32 + j * 8);
                u32x4_t o;
                o.x = __builtin_amdgcn_perm(r.z, r.x, 0x05040100u), o.y = __builtin_amdgcn_perm(r.z, r.x, 0x07060302u);
                o.z = __builtin_amdgcn_perm(r.w, r.y, 0x05040100u), o.w = __builtin_amdgcn_perm(r.w, r.y, 0x07060302u);
                xv[xr][c][j] = o;
                sa = dot2(o.x, 0x3C003C00u, sa), sb = dot2(o.y, 0x3C003C00u, sb);
                sa = dot2(o.z, 0x3C003C00u, sa), sb = dot2(o.w, 0x3C003C00u, sb);
            }
            cr[xr][c] = 1032.0f * sa + 72.0f * sb;
        }
    }

    // part[wave][(row of the workgroup) NR + xr]: slot t holds rows R t .. R t + R - 1 of the workgroup
    auto consume = [&](const Slot &s, int t) {
        float acc[R * NR];
#pragma unroll
        for (int v = 0; v < R * NR; ++v) acc[v] = 0.0f;
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
#pragma unroll
            for (int c = 0; c < NG; ++c) {
                const float scv = on[c] ? h2f(s.sc[rr * NG + c]) : 0.0f;
                if constexpr (NR == 1) {
                    acc[rr] += scv * group_dot_r(s.w[rr * NG + c], xv[0][c], cr[0][c]);
                } else {                                               // the sixteen decoded pairs of the group once, a dot product per row of x
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
        }
        if constexpr (NR > 1) {
            const float r = reduce_many<R * NR>(acc, lane);            // lane l: the total of value l % (R NR)
            if (lane < R * NR) part[wave][t * (R * NR) + lane] = r;
        } else if (R == 2) {
            const float r = reduce2(acc[0], acc[R - 1], lane);         // lane l: row l & 1 of the pair
            if (lane < 2) part[wave][2 * t + lane] = r;
        } else {
            const float r = reduce1(acc[0]);
            if (lane == 0) part[wave][t] = r;
        }
    };
    // two slots in flight; every trip consumes and refills both (refills past the end re-read the last row and are never used;
    // with an odd count of slots the last trip's second consume writes a slot of `part` that nothing reads)
    const int ns = (2 / R) * mine;
#pragma unroll 1
    for (int t = 0; t < ns; t += 2) {
        consume(sl[0], t);
        slot_load(sl[0], t + 2);
        consume(sl[1], t + 1);
        slot_load(sl[1], t + 3);
    }
    wg_barrier();
    if (tid < mine) {
#pragma unroll
        for (int xr = 0; xr < NR; ++xr) {
            const int ia = (2 * tid) * NR + xr, ib = (2 * tid + 1) * NR + xr;
            const float va = (part[0][ia] + part[1][ia]) + (part[2][ia] + part[3][ia]);
            const float vb = (part[0][ib] + part[1][ib]) + (part[2][ib] + part[3][ib]);
            if (i0 + xr < a.n) epi_store<EPI>(a, i0 + xr, RowInfo{0, 0, 0}, wg + tid * W, va, vb, pre[xr]);
        }
    }
}

template <int EPI>
hipError_t launch_long(const GemvArgs &a_in, hipStream_t stream)
{
    GemvArgs a = a_in;
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 1) v = 256;
        cus = v;
    }
    const int U = (a.m + 1) / 2;
    const int chunks = (a.k + 2047) / 2048;                        // 5 .. 16
    // rows of x per pass: four where a lane's x is 32 registers per row (two chunks per wavefront), two beyond
    const int nr = a.n < 2 ? 1 : (chunks <= 8 && a.n >= 3) ? 4 : 2;
    const int passes = (a.n + nr - 1) / nr;
    int gx = std::max(1, cus / std::min(passes, 8));               // one workgroup per CU, shared between the passes
    gx = std::min(gx, U);
    gx = std::max(gx, (U + kLongMaxUnits - 1) / kLongMaxUnits);
    a.units_div = U / gx, a.units_mod = U % gx;
    const dim3 grid(gx, passes);
#define RELAX_LONG(NG_, R_, NR_) hipLaunchKernelGGL((gemv_q4_long_kernel<EPI, NG_, R_, NR_>), grid, dim3(kRThreads), 0, stream, a)
    if (chunks <= 8) {
        if (nr == 4) RELAX_LONG(2, 2, 4);
        else if (nr == 2) RELAX_LONG(2, 2, 2);
        else RELAX_LONG(2, 2, 1);
    } else if (chunks <= 12) {
        if (nr == 2) RELAX_LONG(3, 1, 2);
        else RELAX_LONG(3, 1, 1);
    } else {
        if (nr == 2) RELAX_LONG(4, 1, 2);
        else RELAX_LONG(4, 1, 1);
    }
#undef RELAX_LONG
    return hipGetLastError();
}

}  // namespace

// plain prologue, row-pair epilogue, whole groups, rows of 12289 .. 32768 columns (from two rows of x on: 8193 .. 32768, where
// the one-wavefront-per-row kernel has no room for a second row of x), 16-byte aligned rows of q and x
bool gemv_long_eligible(const GemvArgs &a, int xmode, int epi)
{
    return xmode == X_F16 && (epi == EPI_F16 || epi == EPI_RESID_F16 || epi == EPI_RESID_F32) && a.k > (a.n >= 2 ? 4 : 6) * 2048 && a.k <= 16 * 2048 &&
           (a.k % kGroup == 0) && ((a.k / 8) % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.q) & 15) == 0) &&
           ((reinterpret_cast<uintptr_t>(a.x) & 15) == 0) && a.m >= 2 && a.n >= 1;
}

hipError_t launch_gemv_long(const GemvArgs &a, int epi, hipStream_t stream)
{
    if (epi == EPI_F16) return launch_long<EPI_F16>(a, stream);
    if (epi == EPI_RESID_F16) return launch_long<EPI_RESID_F16>(a, stream);
    if (epi == EPI_RESID_F32) return launch_long<EPI_RESID_F32>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace relax
