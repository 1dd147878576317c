// 3-bit weights (Sec. 5.3 deploys 3-bit models where memory is short): matrix-vector product with the decode in the
// loop, and the dense decode export for the bit-exactness test.
//
// Format: groups of 32 columns share an fp16 scale; the 32 codes u in 0..7 of a group are laid end to end, 3 bits each,
// in three little-endian uint32 words (code c at bits 3c..3c+2 of the 96-bit string; codes 10 and 21 straddle a word
// boundary); weight = (u - 4) * scale.  q: uint32 [m][3k/32], s: fp16 [m][k/32].
//
// Kernel: HBM-bound streaming of q and s, x in registers.  A lane owns the same column groups (lane, lane + 64, ...) for
// every matrix row, so it loads its x values once and keeps them as fp16 pairs; a wavefront then walks matrix rows,
// one row per trip, reading 12 bytes + one scale per lane and group (consecutive lanes read consecutive 12-byte
// groups), with the next row's words requested before the current row is decoded.  Decode uses the fp16 offset trick of
// the 4-bit kernels: 0x6400 | u is the half 1024 + u, two codes of a 6-bit window become one packed pair
// (v & 7) | ((v & 0x38) << 13) | 0x64006400 that goes straight into v_dot2_f32_f16, and the offset leaves per group as
// 1028 * sum(x) (exact for integer-valued x, ~1e-5 relative otherwise).
#include "q4_device.h"

namespace relax {
namespace {

constexpr int kQ3Threads = 256, kQ3Waves = kQ3Threads / kWave;
constexpr int kQ3MaxGroupsPerLane = 6;                       // k <= 6 * 64 * 32 = 12288

// 6-bit window holding codes 2p and 2p+1 of a group
template <int P>
__device__ inline uint32_t window6(uint32_t w0, uint32_t w1, uint32_t w2)
{
    constexpr int bit = 6 * P, word = bit >> 5, sh = bit & 31;
    const uint32_t lo = word == 0 ? w0 : word == 1 ? w1 : w2;
    if constexpr (sh <= 26) return lo >> sh;
    else {
        const uint32_t hi = word == 0 ? w1 : w2;
        return __builtin_amdgcn_alignbit(hi, lo, sh);
    }
}

template <int P>
__device__ inline float pair_dot(uint32_t w0, uint32_t w1, uint32_t w2, const uint32_t *xp, float acc)
{
    const uint32_t v = window6<P>(w0, w1, w2);
    const uint32_t pk = (v & 7u) | ((v & 0x38u) << 13) | 0x64006400u;       // (1024 + u[2P], 1024 + u[2P+1]) as fp16 pair
    return dot2(pk, xp[P], acc);
}

// sum_c x_c * (1024 + u_c) over one group; xp: the group's 32 x values as 16 fp16 pairs in column order
__device__ inline float group_dot3(uint32_t w0, uint32_t w1, uint32_t w2, const uint32_t *xp)
{
    float a = 0.0f, b = 0.0f;
    a = pair_dot<0>(w0, w1, w2, xp, a), b = pair_dot<1>(w0, w1, w2, xp, b);
    a = pair_dot<2>(w0, w1, w2, xp, a), b = pair_dot<3>(w0, w1, w2, xp, b);
    a = pair_dot<4>(w0, w1, w2, xp, a), b = pair_dot<5>(w0, w1, w2, xp, b);
    a = pair_dot<6>(w0, w1, w2, xp, a), b = pair_dot<7>(w0, w1, w2, xp, b);
    a = pair_dot<8>(w0, w1, w2, xp, a), b = pair_dot<9>(w0, w1, w2, xp, b);
    a = pair_dot<10>(w0, w1, w2, xp, a), b = pair_dot<11>(w0, w1, w2, xp, b);
    a = pair_dot<12>(w0, w1, w2, xp, a), b = pair_dot<13>(w0, w1, w2, xp, b);
    a = pair_dot<14>(w0, w1, w2, xp, a), b = pair_dot<15>(w0, w1, w2, xp, b);
    return a + b;
}

struct Q3Row {
    uint32_t w[kQ3MaxGroupsPerLane][3];
    uint16_t s[kQ3MaxGroupsPerLane];
};

template <int J>
__device__ inline void q3_load(Q3Row &r, const uint32_t *q, const uint16_t *s, size_t row, int G, int lane)
{
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int g = lane + kWave * j;
        if (g < G) {
            const uint32_t *p = q + (row * G + g) * 3;
            r.w[j][0] = p[0], r.w[j][1] = p[1], r.w[j][2] = p[2];
            r.s[j] = s[row * G + g];
        }
    }
}

// out[i, r] = sum_k x[i, k] * W[r, k]; grid = (row blocks, n); a wavefront owns rows wave_global, wave_global + W, ...
template <int J>
__global__ __launch_bounds__(kQ3Threads) void gemv_q3_kernel(const uint16_t *__restrict__ x, const uint32_t *__restrict__ q,
                                                             const uint16_t *__restrict__ s, uint16_t *__restrict__ out, int m, int k)
{
    const int G = k >> 5, lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int i = blockIdx.y;
    uint32_t xp[J][16];
    float corr[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
        const int g = lane + kWave * j;
        float sum = 0.0f;
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            uint4 raw = make_uint4(0u, 0u, 0u, 0u);
            if (g < G) raw = *(const uint4 *)(x + (size_t)i * k + (size_t)g * 32 + v4 * 8);
            xp[j][4 * v4] = raw.x, xp[j][4 * v4 + 1] = raw.y, xp[j][4 * v4 + 2] = raw.z, xp[j][4 * v4 + 3] = raw.w;
        }
#pragma unroll
        for (int p = 0; p < 16; ++p) sum = dot2(0x3C003C00u, xp[j][p], sum);        // (1, 1) . (x[2p], x[2p+1])
        corr[j] = 1028.0f * sum;
    }
    const int W = gridDim.x * kQ3Waves;
    int r = blockIdx.x * kQ3Waves + wave;
    Q3Row cur, nxt;
    if (r < m) q3_load<J>(cur, q, s, (size_t)r, G, lane);
    for (; r < m; r += W) {
        if (r + W < m) q3_load<J>(nxt, q, s, (size_t)(r + W), G, lane);
        float acc = 0.0f;
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int g = lane + kWave * j;
            if (g < G) acc += h2f(cur.s[j]) * (group_dot3(cur.w[j][0], cur.w[j][1], cur.w[j][2], xp[j]) - corr[j]);
        }
        acc = wave_sum(acc);
        if (lane == 0) out[(size_t)i * m + r] = f2h(acc);
        cur = nxt;
    }
}

__global__ void unpack_q3_kernel(const uint32_t *q, int8_t *out, int m, int k)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)m * k) return;
    const size_t row = e / k;
    const int c = (int)(e - row * k), g = c >> 5, bit = 3 * (c & 31);
    const uint32_t *p = q + (row * (k >> 5) + g) * 3;
    const int word = bit >> 5, sh = bit & 31;
    uint32_t v = p[word] >> sh;
    if (sh > 29) v |= p[word + 1] << (32 - sh);
    out[e] = (int8_t)((int)(v & 7u) - 4);
}

// ---- native 3-bit layout: the same 96 bits per group, placed so that one v_and_or_b32 yields a ready fp16 pair ----------
// Canonical codes lie end to end; a 6-bit window has to be shifted into place for every pair (about five vector ops per
// two weights, which made the 3-bit matvec slower than the 4-bit one although it reads fewer bytes).  relax_repack_q3
// rewrites a matrix once into this layout of a group's three words (columns c = 0..31 of the group, code u_c):
//   word w (0..2), position j (0..4): u_{2(5w+j)} in bits 3j..3j+2, u_{2(5w+j)+1} in bits 16+3j..16+3j+2
//   (the 15 pairs of columns 0..29: pair p = 5w + j, its even column in the low half-word, its odd column in the high one);
//   bit i (0..2) of u_30 is bit 15 of word i, bit i of u_31 is bit 31 of word i.
// (v & 0x00070007) | 0x64006400 is then the fp16 pair (1024 + u_even, 1024 + u_odd) of position 0, the masks 0x00380038 and
// 0x01C001C0 give (1024 + 8u, ...) and (1024 + 64u, ...) of positions 1 and 2 without a shift -- all inside the ten mantissa
// bits -- and positions 3, 4 are positions 0, 1 of v >> 9.  Pairs of the three scale classes go to three accumulators;
// sum x (u - 4) = A + B / 8 + C / 64 - (1028 sum_A x + 132 sum_B x + 20 sum_C x), the bracket precomputed per group of x.
// 24 decode ops per group, shared by every row of x in the pass, plus 16 dot products per row of x.

// and_or3, q3n_class and q3n_decode (the decode of a group in this layout) live in relax_common.h: the fused one-row kernel
// of the decoder layer uses them too.

// one group: canonical words -> native words
__global__ void repack_q3_kernel(const uint32_t *src, uint32_t *dst, size_t groups)
{
    const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= groups) return;
    const uint32_t a = src[3 * g], b = src[3 * g + 1], c = src[3 * g + 2];
    uint32_t u[32];
#pragma unroll
    for (int col = 0; col < 32; ++col) {
        const int bit = 3 * col, word = bit >> 5, sh = bit & 31;
        const uint32_t lo = word == 0 ? a : word == 1 ? b : c, hi = word == 0 ? b : c;
        uint32_t v = lo >> sh;
        if (sh > 29) v |= hi << (32 - sh);
        u[col] = v & 7u;
    }
    uint32_t o[3] = {0u, 0u, 0u};
#pragma unroll
    for (int p = 0; p < 15; ++p) o[p / 5] |= (u[2 * p] << (3 * (p % 5))) | (u[2 * p + 1] << (16 + 3 * (p % 5)));
#pragma unroll
    for (int i = 0; i < 3; ++i) o[i] |= (((u[30] >> i) & 1u) << 15) | (((u[31] >> i) & 1u) << 31);
    dst[3 * g] = o[0], dst[3 * g + 1] = o[1], dst[3 * g + 2] = o[2];
}

__global__ void unpack_q3n_kernel(const uint32_t *q, int8_t *out, int m, int k)
{
    const size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (size_t)m * k) return;
    const size_t row = e / k;
    const int c = (int)(e - row * k), g = c >> 5, col = c & 31;
    const uint32_t *p = q + (row * (k >> 5) + g) * 3;
    uint32_t u;
    if (col < 30) {
        const int pr = col >> 1;
        u = (p[pr / 5] >> (3 * (pr % 5) + 16 * (col & 1))) & 7u;
    } else {
        const int sh = col == 30 ? 15 : 31;
        u = ((p[0] >> sh) & 1u) | (((p[1] >> sh) & 1u) << 1) | (((p[2] >> sh) & 1u) << 2);
    }
    out[e] = (int8_t)((int)u - 4);
}

constexpr int kQ3nRows = 2;                                  // matrix rows per slot; two slots in flight per wavefront

// out[i0 + xr, r] for NR rows of x per pass: grid = (workgroups, passes).  A wavefront owns the row pairs wg, wg + W, ...
template <int J, int NR>
__global__ __launch_bounds__(kQ3Threads) void gemv_q3n_kernel(const uint16_t *__restrict__ x, const uint32_t *__restrict__ q,
                                                              const uint16_t *__restrict__ s, uint16_t *__restrict__ out, int m, int k, int n)
{
    const int G = k >> 5, lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int i0 = blockIdx.y * NR;
    // the lane's x values of every row of the pass, as fp16 pairs in column order, and the offset term of each group
    uint32_t xp[NR][J][16];
    float corr[NR][J];
#pragma unroll
    for (int xr = 0; xr < NR; ++xr) {
        const int i = min(i0 + xr, n - 1);                   // a ragged last pass re-reads the last row (never stored)
#pragma unroll
        for (int j = 0; j < J; ++j) {
            const int g = min(lane + kWave * j, G - 1);
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const uint4 raw = *(const uint4 *)(x + (size_t)i * k + (size_t)g * 32 + v4 * 8);
                xp[xr][j][4 * v4] = raw.x, xp[xr][j][4 * v4 + 1] = raw.y, xp[xr][j][4 * v4 + 2] = raw.z, xp[xr][j][4 * v4 + 3] = raw.w;
            }
        }
    }
    bool on[J];
#pragma unroll
    for (int j = 0; j < J; ++j) on[j] = lane + kWave * j < G;

    struct Slot {
        uint32_t w[kQ3nRows][J][3];
        uint16_t sc[kQ3nRows][J];
    };
    const int U = (m + kQ3nRows - 1) / kQ3nRows;             // row pairs
    const int W = gridDim.x * kQ3Waves, wg = blockIdx.x * kQ3Waves + wave;
    auto slot_load = [&](Slot &sl, int u) {                  // unit u; past the end: the last unit again (dropped)
        __builtin_amdgcn_sched_barrier(0);                   // the requests of a slot stay together, where they are written
        u = min(u, U - 1);
#pragma unroll
        for (int rr = 0; rr < kQ3nRows; ++rr) {
            const size_t row = (size_t)min(u * kQ3nRows + rr, m - 1);
#pragma unroll
            for (int j = 0; j < J; ++j) {
                const int g = min(lane + kWave * j, G - 1);
                const uint32_t *p = q + (row * G + g) * 3;
                sl.w[rr][j][0] = stream_load(p), sl.w[rr][j][1] = stream_load(p + 1), sl.w[rr][j][2] = stream_load(p + 2);
                sl.sc[rr][j] = s[row * G + g];
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    // both slots are requested before anything waits for x
    Slot a, b;
    slot_load(a, wg);
    slot_load(b, wg + W);
#pragma unroll
    for (int xr = 0; xr < NR; ++xr)
#pragma unroll
        for (int j = 0; j < J; ++j) {
            float sc[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int p = 0; p < 16; ++p) sc[q3n_class(p)] = dot2(0x3C003C00u, xp[xr][j][p], sc[q3n_class(p)]);
            corr[xr][j] = 1028.0f * sc[0] + 132.0f * sc[1] + 20.0f * sc[2];
        }
    // the dot products of a slot; its registers are free afterwards, so the next request goes out before the reduction
    auto dots = [&](const Slot &sl, float *tot) {
#pragma unroll
        for (int rr = 0; rr < kQ3nRows; ++rr) {
#pragma unroll
            for (int xr = 0; xr < NR; ++xr) tot[rr * NR + xr] = 0.0f;
#pragma unroll
            for (int j = 0; j < J; ++j) {
                uint32_t pk[16];
                q3n_decode(sl.w[rr][j][0], sl.w[rr][j][1], sl.w[rr][j][2], pk);
                const float scale = on[j] ? h2f(sl.sc[rr][j]) : 0.0f;
#pragma unroll
                for (int xr = 0; xr < NR; ++xr) {
                    float acc[3] = {0.0f, 0.0f, 0.0f};
#pragma unroll
                    for (int p = 0; p < 16; ++p) acc[q3n_class(p)] = dot2(pk[p], xp[xr][j][p], acc[q3n_class(p)]);
                    tot[rr * NR + xr] += scale * (acc[0] + acc[1] * 0.125f + acc[2] * 0.015625f - corr[xr][j]);
                }
            }
        }
    };
    auto finish = [&](float *tot, int u) {
        const float r = reduce_many<kQ3nRows * NR>(tot, lane);
        if (u < U && lane < kQ3nRows * NR) {                 // lane l: row l / NR of the unit, x row l % NR of the pass
            const int row = u * kQ3nRows + lane / NR, i = i0 + lane % NR;
            if (row < m && i < n) out[(size_t)i * m + row] = f2h(r);
        }
    };
    for (int u = wg; u < U; u += 2 * W) {
        float ta[kQ3nRows * NR], tb[kQ3nRows * NR];
        dots(a, ta);
        slot_load(a, u + 2 * W);
        finish(ta, u);
        dots(b, tb);
        slot_load(b, u + 3 * W);
        finish(tb, u + W);
    }
}

}  // namespace

bool gemv_q3_supported(int m, int k) { return m >= 1 && k >= 32 && k % 32 == 0 && k <= kQ3MaxGroupsPerLane * kWave * 32; }

hipError_t launch_gemv_q3(const uint16_t *x, const relax_qmat &w, int n, uint16_t *out, hipStream_t stream)
{
    const int G = w.k / 32, J = (G + kWave - 1) / kWave;
    (void)hipGetLastError();               // an error another library left on this thread is not this launch's
    // about two workgroups per CU keep eight wavefronts per CU streaming; never more workgroups than row quadruples
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    const int blocks = std::max(1, std::min((w.m + kQ3Waves - 1) / kQ3Waves, 4 * cus));
    const dim3 grid(blocks, n), block(kQ3Threads);
    const uint32_t *q = static_cast<const uint32_t *>(w.q);
    const uint16_t *s = static_cast<const uint16_t *>(w.s);
    switch (J) {
    case 1: hipLaunchKernelGGL(gemv_q3_kernel<1>, grid, block, 0, stream, x, q, s, out, w.m, w.k); break;
    case 2: hipLaunchKernelGGL(gemv_q3_kernel<2>, grid, block, 0, stream, x, q, s, out, w.m, w.k); break;
    case 3: hipLaunchKernelGGL(gemv_q3_kernel<3>, grid, block, 0, stream, x, q, s, out, w.m, w.k); break;
    case 4: hipLaunchKernelGGL(gemv_q3_kernel<4>, grid, block, 0, stream, x, q, s, out, w.m, w.k); break;
    case 5: hipLaunchKernelGGL(gemv_q3_kernel<5>, grid, block, 0, stream, x, q, s, out, w.m, w.k); break;
    case 6: hipLaunchKernelGGL(gemv_q3_kernel<6>, grid, block, 0, stream, x, q, s, out, w.m, w.k); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_unpack_q3(const relax_qmat &w, int8_t *out, hipStream_t stream)
{
    const size_t total = (size_t)w.m * w.k;
    (void)hipGetLastError();
    hipLaunchKernelGGL(unpack_q3_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, static_cast<const uint32_t *>(w.q), out, w.m, w.k);
    return hipGetLastError();
}

// x rows per pass of the native-layout kernel: as many as the registers of a lane hold next to the slots
int gemv_q3n_rows_per_pass(int k, int n)
{
    const int J = (k / 32 + kWave - 1) / kWave;
    const int cap = J <= 2 ? 4 : J <= 4 ? 2 : 1;
    return n >= 4 && cap >= 4 ? 4 : n >= 2 && cap >= 2 ? 2 : 1;
}

template <int J, int NR>
static void launch_q3n(const uint16_t *x, const uint32_t *q, const uint16_t *s, uint16_t *out, int m, int k, int n, int blocks, hipStream_t stream)
{
    hipLaunchKernelGGL((gemv_q3n_kernel<J, NR>), dim3(blocks, (n + NR - 1) / NR), dim3(kQ3Threads), 0, stream, x, q, s, out, m, k, n);
}

hipError_t launch_gemv_q3_native(const uint16_t *x, const relax_qmat &w, int n, uint16_t *out, hipStream_t stream)
{
    if (n == 1) {                                // one row: the 3-bit stream of the decode layer's matvec kernel (x staged once per
        GemvArgs a = {};                         // workgroup, one workgroup per CU) is 1 to 1.5 us faster per launch than the kernel below
        a.x = x, a.q = static_cast<const uint32_t *>(w.q), a.s = static_cast<const uint16_t *>(w.s), a.m = w.m, a.k = w.k, a.n = 1;
        a.out_f16 = out;
        if (gemv_q3w_eligible(a)) return launch_gemv_q3w(a, X_F16, EPI_F16, stream);
    }
    const int G = w.k / 32, J = (G + kWave - 1) / kWave, NR = gemv_q3n_rows_per_pass(w.k, n);
    (void)hipGetLastError();
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    }
    const int units = (w.m + kQ3nRows - 1) / kQ3nRows;
    // two workgroups per CU, one for the two variants whose registers leave room for a single one
    const int per_cu = (J == 6 || (J == 4 && NR == 2)) ? 1 : 2;
    const int blocks = std::max(1, std::min((units + kQ3Waves - 1) / kQ3Waves, per_cu * cus));
    const uint32_t *q = static_cast<const uint32_t *>(w.q);
    const uint16_t *s = static_cast<const uint16_t *>(w.s);
#define RELAX_Q3N(JJ, RR) launch_q3n<JJ, RR>(x, q, s, out, w.m, w.k, n, blocks, stream)
    switch (J * 8 + NR) {
    case 1 * 8 + 1: RELAX_Q3N(1, 1); break;
    case 1 * 8 + 2: RELAX_Q3N(1, 2); break;
    case 1 * 8 + 4: RELAX_Q3N(1, 4); break;
    case 2 * 8 + 1: RELAX_Q3N(2, 1); break;
    case 2 * 8 + 2: RELAX_Q3N(2, 2); break;
    case 2 * 8 + 4: RELAX_Q3N(2, 4); break;
    case 3 * 8 + 1: RELAX_Q3N(3, 1); break;
    case 3 * 8 + 2: RELAX_Q3N(3, 2); break;
    case 4 * 8 + 1: RELAX_Q3N(4, 1); break;
    case 4 * 8 + 2: RELAX_Q3N(4, 2); break;
    case 5 * 8 + 1: RELAX_Q3N(5, 1); break;
    case 6 * 8 + 1: RELAX_Q3N(6, 1); break;
    default: return hipErrorInvalidValue;
    }
#undef RELAX_Q3N
    return hipGetLastError();
}

hipError_t launch_repack_q3(const relax_qmat &w, uint32_t *dst, hipStream_t stream)
{
    const size_t groups = (size_t)w.m * (w.k / 32);
    (void)hipGetLastError();
    hipLaunchKernelGGL(repack_q3_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, stream, static_cast<const uint32_t *>(w.q), dst, groups);
    return hipGetLastError();
}

hipError_t launch_unpack_q3_native(const relax_qmat &w, int8_t *out, hipStream_t stream)
{
    const size_t total = (size_t)w.m * w.k;
    (void)hipGetLastError();
    hipLaunchKernelGGL(unpack_q3n_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, static_cast<const uint32_t *>(w.q), out, w.m, w.k);
    return hipGetLastError();
}

}  // namespace relax
