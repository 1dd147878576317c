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

}  // namespace relax
