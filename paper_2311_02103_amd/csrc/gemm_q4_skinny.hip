// Fused int4-decode matmul for a few rows (2 <= n <= 64: batched decode, short prefills):
//   out[i,r] = sum_c x[i,c] * (u(r,c) - 8) * s[r, c/32].
//
// With few rows the contraction is still bound by the one pass over the packed weights (Relax, Sec. 5.1:
// batch sizes between the matrix-vector case and the compute-bound GEMM), but every weight now meets n
// activations, so the products go to the matrix cores.  Mapping for gfx950:
//   - v_mfma_f32_32x32x16_f16 with the weights as the A operand straight from global memory: lane l of a
//     wavefront owns weight row (l % 32) and one half (l / 32) of each 256-wide k round, i.e. 64 contiguous bytes
//     of packed codes per round (four 16-byte loads) and four group scales; each word is decoded in registers
//     (the exact offset-removal decode of the large-n GEMM) into the eight fp16 values of one MFMA k step.
//     Nothing of the weight stream goes through LDS; loads run two rounds ahead of their use.
//   - The order of k inside an MFMA is free as long as A and B agree: k step s of half hf pairs word 16 hf + s of
//     the round with the matching 8-wide x packet.  The x chunk of a round (n rows x 256) is staged in LDS once per
//     workgroup, each packet in the order [x0 x4 x1 x5 x2 x6 x3 x7] of the decode, and shared by the four
//     wavefronts (four 32-row blocks of weight rows).  Columns of the 32-wide MFMA tile beyond n are never stored.
//   - m x k is cut into workgroup tasks of 128 weight rows x one k range (split-K) so that the grid fills 256 CUs
//     several times over even when m is small; every task writes its fp32 partial tile to the workspace and a small
//     finishing kernel adds the partials IN A FIXED ORDER and applies the epilogue (plain fp16, residual adds,
//     SwiGLU).  No atomics: results are reproducible run to run.
#include <atomic>

#include "relax_common.h"

namespace relax {

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kRound = 256;                  // k granule every matrix has to be a multiple of (a round is 256 or 128 columns)
constexpr int kRowsPerBlock = 128;           // 4 wavefronts x 32 weight rows
constexpr int kMaxRounds = 16;               // rounds per task at most (the task's scales sit in LDS: 128 rows x 16 bytes per round)

__device__ __forceinline__ uint32_t pk_add(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, a) + __builtin_bit_cast(half2_t, b));
}
__device__ __forceinline__ uint32_t pk_mul(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, a) * __builtin_bit_cast(half2_t, b));
}
__device__ __forceinline__ uint32_t pk_fma(uint32_t a, uint32_t b, uint32_t c)
{
    half2_t r = __builtin_elementwise_fma(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), __builtin_bit_cast(half2_t, c));
    return __builtin_bit_cast(uint32_t, r);
}
// (w & mask) | bits as one VALU op (mask from a scalar register, bits from a vector register)
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t bits)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(bits));
    return r;
}
// one packed word and its group scale (fp16 pair s,s) -> 8 fp16 weights in the order [e0 e4 e1 e5 e2 e6 e3 e7];
// exact up to the final multiply: 1024+u-1032, (1024+16u)/16-72
__device__ __forceinline__ half8_t decode_word(uint32_t w, uint32_t s2)
{
    const uint32_t w8 = w >> 8;
    const uint32_t a0 = and_or(w, 0x000F000Fu, 0x64006400u), a1 = and_or(w, 0x00F000F0u, 0x64006400u);
    const uint32_t a2 = and_or(w8, 0x000F000Fu, 0x64006400u), a3 = and_or(w8, 0x00F000F0u, 0x64006400u);
    const uint32_t kNeg1032 = 0xE408E408u, kSixteenth = 0x2C002C00u, kNeg72 = 0xD480D480u;
    u32x4_t r;
    r.x = pk_mul(pk_add(a0, kNeg1032), s2);
    r.y = pk_mul(pk_fma(a1, kSixteenth, kNeg72), s2);
    r.z = pk_mul(pk_add(a2, kNeg1032), s2);
    r.w = pk_mul(pk_fma(a3, kSixteenth, kNeg72), s2);
    return __builtin_bit_cast(half8_t, r);
}

struct SkinnyArgs {
    const uint16_t *x;       // [n,k] fp16
    const uint32_t *q;       // [m,k/8]
    const uint16_t *s;       // [m, k / (32 << gshift)]
    int32_t gshift;          // quantisation group = 32 << gshift columns
    float *partial;          // [splits][n][m] fp32
    int32_t n, m, k;
    int32_t rounds_per_split;
};

// grid: x = 128-row tile of weight rows, y = k split.  NF = 32-wide column blocks of the MFMA tile, XR = x rows kept
// in LDS (n <= XR <= 32 NF).  MFMA columns beyond n compute on whatever the LDS rows hold (for XR = 16 the lanes of
// columns 16..31 re-read rows 0..15) and are never stored: a column of the result depends on its own x row only.
template <int NF, int XR, int KR>
__global__ __launch_bounds__(256) void skinny_q4_kernel(SkinnyArgs a)
{
    constexpr int kXPitch = KR + 8;                       // LDS row pitch of the x chunk in halfs (16-byte fragment reads of 32 rows hit distinct banks)
    constexpr int W = KR / 16;                            // packed words (= MFMA k steps) per lane and round: the lane's half of the round
    constexpr int XP = XR * (KR / 8) / 256;               // 16-byte x packets a thread stages per round
    constexpr int kXBuf = XR * kXPitch;
    extern __shared__ __align__(16) uint16_t lds[];       // x chunks [2][XR][kXPitch], then the scale tile [128][sc_pitch]
    uint16_t *const xs = lds, *const scs = lds + 2 * kXBuf;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row32 = lane & 31, hf = lane >> 5;
    const int kw = a.k >> 3, SG = a.k >> (5 + a.gshift);   // packed words and scales per weight row
    const int total_rounds = a.k / KR;
    const int r_begin = blockIdx.y * a.rounds_per_split, r_end = min(total_rounds, r_begin + a.rounds_per_split);
    const int nr = r_end - r_begin;                       // >= 1 by construction of the grid
    const int spr = a.rounds_per_split * KR / 256;        // 16-byte scale packets (8 groups = 256 columns) per row of the task
    const int sc_pitch = spr * 8 + 8;                     // halfs per row of the scale tile (+16 bytes: rows start in different banks)

    // ---- group scales of the whole task, once: 128 rows x (8 nr) fp16, 16-byte packets, coalesced along each row ----
    // (per-round 8-byte loads would touch every 128-byte line of the scale rows eight rounds in a row)
    // The tile always holds one entry per 32 columns; with a wider quantisation group a packet's 8 entries are 4 or 2
    // scales of the matrix, each written twice or four times (8- or 4-byte loads: k % 256 == 0 keeps them aligned).
    u32x4_t screg[kMaxRounds / 2];
#pragma unroll
    for (int i = 0; i < kMaxRounds / 2; ++i) {
        const int pk = tid + i * 256, row = pk / spr, pp = pk - row * spr;
        const int grow = min(blockIdx.x * kRowsPerBlock + min(row, kRowsPerBlock - 1), a.m - 1);
        const size_t sub = (size_t)r_begin * (KR / 32) + (size_t)min(pp, nr * KR / 256 - 1) * 8;      // first 32-column sub-group of the packet
        const uint16_t *src = a.s + (size_t)grow * SG + (sub >> a.gshift);
        if (a.gshift == 0) {
            screg[i] = *(const u32x4_t *)src;
        } else if (a.gshift == 1) {
            const u32x2_t four = *(const u32x2_t *)src;                                                // s0 s1 | s2 s3
            screg[i] = u32x4_t{__builtin_amdgcn_perm(four.x, four.x, 0x01000100u), __builtin_amdgcn_perm(four.x, four.x, 0x03020302u),
                               __builtin_amdgcn_perm(four.y, four.y, 0x01000100u), __builtin_amdgcn_perm(four.y, four.y, 0x03020302u)};
        } else {
            const uint32_t two = *(const uint32_t *)src;                                               // s0 s1
            const uint32_t lo = __builtin_amdgcn_perm(two, two, 0x01000100u), hi = __builtin_amdgcn_perm(two, two, 0x03020302u);
            screg[i] = u32x4_t{lo, lo, hi, hi};
        }
    }

    const int wrow = min(blockIdx.x * kRowsPerBlock + wave * 32 + row32, a.m - 1);
    const uint32_t *qsrc = a.q + (size_t)wrow * kw + (size_t)r_begin * (KR / 8) + hf * W;
    // x staging roles: packet pk = tid + p * 256 -> x row pk / (KR/8), packet pk % (KR/8) of the round
    const uint16_t *xsrc[XP];
    bool xon[XP];
#pragma unroll
    for (int p = 0; p < XP; ++p) {
        const int pk = tid + p * 256, xr = pk / (KR / 8);
        xon[p] = xr < a.n;
        xsrc[p] = a.x + (size_t)min(xr, a.n - 1) * a.k + (size_t)r_begin * KR + (pk % (KR / 8)) * 8;
    }

    // Registers of one round in flight: the thread's share of the x chunk and the lane's 64 bytes of codes.
    // Memory operations of a wavefront complete in order, so x goes first: the chunk is needed one round before the codes.
    struct Stage {
        u32x4_t x[XP];
        u32x4_t w[W / 4];
    };
    auto stage_load = [&](Stage &S, int r) {              // r relative to r_begin, clamped: the tail re-reads the last round
        r = min(r, nr - 1);
#pragma unroll
        for (int p = 0; p < XP; ++p) S.x[p] = *(const u32x4_t *)(xsrc[p] + (size_t)r * KR);
#pragma unroll
        // (plain loads: the four 16-byte pieces of a lane's 64 bytes and its neighbour's share 128-byte lines, which have to stay cached between them)
        for (int i = 0; i < W / 4; ++i) S.w[i] = *(const u32x4_t *)(qsrc + (size_t)r * (KR / 8) + i * 4);
    };
    auto x_store = [&](const Stage &S, int buf) {
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            if (!xon[p]) continue;
            const int pk = tid + p * 256;
            // [x0 x1 | x2 x3 | x4 x5 | x6 x7] -> [x0 x4 | x1 x5 | x2 x6 | x3 x7]
            u32x4_t o;
            o.x = __builtin_amdgcn_perm(S.x[p].z, S.x[p].x, 0x05040100u);
            o.y = __builtin_amdgcn_perm(S.x[p].z, S.x[p].x, 0x07060302u);
            o.z = __builtin_amdgcn_perm(S.x[p].w, S.x[p].y, 0x05040100u);
            o.w = __builtin_amdgcn_perm(S.x[p].w, S.x[p].y, 0x07060302u);
            *(u32x4_t *)(xs + buf * kXBuf + (pk / (KR / 8)) * kXPitch + (pk % (KR / 8)) * 8) = o;
        }
    };
    auto lds_barrier = [&]() {                            // LDS only: global loads stay in flight across it
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    float16_t acc[NF];
#pragma unroll
    for (int j = 0; j < NF; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;

    // one round: W k steps; word W hf + s of the lane's codes against x packet W hf + s of the chunk
    const uint16_t *sc_lane = scs + (wave * 32 + row32) * sc_pitch + hf * (W / 4);
    auto round = [&](const Stage &S, int r, int buf) {
        const uint16_t *xb = xs + buf * kXBuf + (row32 & (XR - 1)) * kXPitch + hf * (KR / 2);
        // the group scales of the lane's half (W/4 of them), each duplicated into both halves of a register
        u32x2_t sc;
        if (W == 16) sc = *(const u32x2_t *)(sc_lane + r * 8);
        else sc = u32x2_t{*(const uint32_t *)(sc_lane + r * 4), 0u};
        const uint32_t s2[4] = {__builtin_amdgcn_perm(sc.x, sc.x, 0x01000100u), __builtin_amdgcn_perm(sc.x, sc.x, 0x03020302u),
                                __builtin_amdgcn_perm(sc.y, sc.y, 0x01000100u), __builtin_amdgcn_perm(sc.y, sc.y, 0x03020302u)};
#pragma unroll
        for (int s = 0; s < W; ++s) {
            const u32x4_t &wv = S.w[s >> 2];
            const uint32_t word = (s & 3) == 0 ? wv.x : (s & 3) == 1 ? wv.y : (s & 3) == 2 ? wv.z : wv.w;
            const half8_t af = decode_word(word, s2[s >> 2]);
#pragma unroll
            for (int j = 0; j < NF; ++j) {
                const half8_t bf = *(const half8_t *)(xb + (XR > 32 ? j * 32 * kXPitch : 0) + s * 8);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf, acc[j], 0, 0, 0);
            }
        }
    };

    // Software pipeline, three register stages: everything of round r+2 is requested at the top of round r; the x chunk
    // of round r+1 moves from registers to LDS at the end of round r.  The loop has one exit: rounds past the end of
    // the k range still load (clamped), store and synchronise, but skip the arithmetic.
    Stage S0, S1, S2;
    stage_load(S0, 0);
    stage_load(S1, 1);
#pragma unroll
    for (int i = 0; i < kMaxRounds / 2; ++i) {
        const int pk = tid + i * 256, row = pk / spr, pp = pk - row * spr;
        if (row < kRowsPerBlock) *(u32x4_t *)(scs + row * sc_pitch + pp * 8) = screg[i];
    }
    x_store(S0, 0);
    lds_barrier();
    for (int r = 0; r < nr; r += 3) {
        stage_load(S2, r + 2);
        round(S0, r, r & 1);
        x_store(S1, (r + 1) & 1);
        lds_barrier();
        stage_load(S0, r + 3);
        if (r + 1 < nr) round(S1, r + 1, (r + 1) & 1);
        x_store(S2, (r + 2) & 1);
        lds_barrier();
        stage_load(S1, r + 4);
        if (r + 2 < nr) round(S2, r + 2, (r + 2) & 1);
        x_store(S0, (r + 3) & 1);
        lds_barrier();
    }

    // partial[split][i][row]: register v of column block j is weight row 8 (v/4) + 4 hf + v%4, x row 32 j + row32
    const int row0 = blockIdx.x * kRowsPerBlock + wave * 32;
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        const int i = j * 32 + row32;
        if (i >= a.n) continue;
        float *dst = a.partial + ((size_t)blockIdx.y * a.n + i) * a.m;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int r = row0 + b * 8 + hf * 4;
            if (r < a.m)                                   // m % 4 == 0 is checked by the launcher
                *(float4_t *)(dst + r) = float4_t{acc[j][b * 4], acc[j][b * 4 + 1], acc[j][b * 4 + 2], acc[j][b * 4 + 3]};
        }
    }
}

// out = epilogue(sum over splits, in order, of partial[s][i][r]); one thread per 4 consecutive r (SwiGLU: 4 gate columns)
template <int EPI>
__global__ __launch_bounds__(256) void skinny_finish_kernel(const float *__restrict__ partial, int splits, int n, int m,
                                                            uint16_t *__restrict__ out_f16, float *__restrict__ out_f32,
                                                            const void *__restrict__ resid)
{
    const int width = EPI == EPI_SWIGLU ? m / 2 : m;
    const size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (idx >= (size_t)n * width) return;
    const int i = (int)(idx / width), r = (int)(idx - (size_t)i * width);
    float4_t sum = {0.0f, 0.0f, 0.0f, 0.0f}, sum2 = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int s = 0; s < splits; ++s) {
        const float *p = partial + ((size_t)s * n + i) * m + r;
        sum += *(const float4_t *)p;
        if (EPI == EPI_SWIGLU) sum2 += *(const float4_t *)(p + width);
    }
    const size_t at = (size_t)i * width + r;
    float v[4] = {sum.x, sum.y, sum.z, sum.w};
    if (EPI == EPI_RESID_F32) {
        const u32x2_t xx = *(const u32x2_t *)((const uint16_t *)resid + at);
        *(float4_t *)(out_f32 + at) = float4_t{h2f((uint16_t)(xx.x & 0xFFFFu)) + v[0], h2f((uint16_t)(xx.x >> 16)) + v[1],
                                               h2f((uint16_t)(xx.y & 0xFFFFu)) + v[2], h2f((uint16_t)(xx.y >> 16)) + v[3]};
        return;
    }
    if (EPI == EPI_RESID_F16) {
        const float4_t rr = *(const float4_t *)((const float *)resid + at);
        v[0] += rr.x, v[1] += rr.y, v[2] += rr.z, v[3] += rr.w;
    }
    if (EPI == EPI_SWIGLU) {
        const float u[4] = {sum2.x, sum2.y, sum2.z, sum2.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = v[e] / (1.0f + __expf(-v[e])) * u[e];
    }
    *(u32x2_t *)(out_f16 + at) = u32x2_t{f2h(v[0]) | ((uint32_t)f2h(v[1]) << 16), f2h(v[2]) | ((uint32_t)f2h(v[3]) << 16)};
}

// ---- finishing kernels that also do the light step that follows the matmul in the layer (Sec. 4.2: the element-wise
// ---- neighbours of a matmul fold into it; here into its finishing pass, one launch less each) ----

__device__ __forceinline__ void sum_splits8(const float *partial, int splits, size_t split_stride, size_t at, float *v)
{
    float4_t a = {0.0f, 0.0f, 0.0f, 0.0f}, b = {0.0f, 0.0f, 0.0f, 0.0f};
    int s = 0;
    for (; s + 4 <= splits; s += 4) {                      // four splits in flight, added in order
        float4_t ta[4], tb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float *p = partial + (size_t)(s + u) * split_stride + at;
            ta[u] = *(const float4_t *)p, tb[u] = *(const float4_t *)(p + 4);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) a += ta[u], b += tb[u];
    }
    for (; s < splits; ++s) {
        const float *p = partial + (size_t)s * split_stride + at;
        a += *(const float4_t *)p;
        b += *(const float4_t *)(p + 4);
    }
    v[0] = a.x, v[1] = a.y, v[2] = a.z, v[3] = a.w, v[4] = b.x, v[5] = b.y, v[6] = b.z, v[7] = b.w;
}
__device__ __forceinline__ void unpack8h(const u32x4_t raw, float *v)
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) v[2 * j] = h2f((uint16_t)(w[j] & 0xFFFFu)), v[2 * j + 1] = h2f((uint16_t)(w[j] >> 16));
}
__device__ __forceinline__ u32x4_t pack8h(const float *v)
{
    return u32x4_t{f2h(v[0]) | ((uint32_t)f2h(v[1]) << 16), f2h(v[2]) | ((uint32_t)f2h(v[3]) << 16),
                   f2h(v[4]) | ((uint32_t)f2h(v[5]) << 16), f2h(v[6]) | ((uint32_t)f2h(v[7]) << 16)};
}

constexpr int kFuseNormPasses = 4;           // rows of up to 4 x 2048 columns stay in registers between the sum and the scaling

// Residual epilogue + RMSNorm of the result, one workgroup per row (m <= 8192, m % 8 == 0):
//   EPI_RESID_F32: y = x(fp16 resid) + sum -> out_f32;             xn = RMSNorm(y) * norm_w
//   EPI_RESID_F16: y = fp16(sum + resid(fp32)) -> out_f16;         xn = RMSNorm(y) * norm_w (of the rounded values: what the next layer reads)
// Same arithmetic, element by element and in the same order, as the plain finishing kernel followed by the row-norm kernel.
template <int EPI>
__global__ __launch_bounds__(1024) void skinny_finish_norm_kernel(const float *__restrict__ partial, int splits, int n, int m,
                                                                 uint16_t *__restrict__ out_f16, float *__restrict__ out_f32,
                                                                 const void *__restrict__ resid, const uint16_t *__restrict__ norm_w,
                                                                 uint16_t *__restrict__ xn, float eps)
{
    __shared__ float red[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i = blockIdx.x, T = blockDim.x;
    const size_t base = (size_t)i * m, split_stride = (size_t)n * m;
    float v[kFuseNormPasses][8];
    float ss = 0.0f;
#pragma unroll
    for (int p = 0; p < kFuseNormPasses; ++p) {
        const int c = (p * T + tid) * 8;
        if (c < m) {
            sum_splits8(partial, splits, split_stride, base + c, v[p]);
            if (EPI == EPI_RESID_F32) {
                float xr[8];
                unpack8h(*(const u32x4_t *)((const uint16_t *)resid + base + c), xr);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[p][e] = xr[e] + v[p][e];
                *(float4_t *)(out_f32 + base + c) = float4_t{v[p][0], v[p][1], v[p][2], v[p][3]};
                *(float4_t *)(out_f32 + base + c + 4) = float4_t{v[p][4], v[p][5], v[p][6], v[p][7]};
            } else {
                const float4_t r0 = *(const float4_t *)((const float *)resid + base + c), r1 = *(const float4_t *)((const float *)resid + base + c + 4);
                v[p][0] += r0.x, v[p][1] += r0.y, v[p][2] += r0.z, v[p][3] += r0.w;
                v[p][4] += r1.x, v[p][5] += r1.y, v[p][6] += r1.z, v[p][7] += r1.w;
                const u32x4_t o = pack8h(v[p]);
                *(u32x4_t *)(out_f16 + base + c) = o;
                unpack8h(o, v[p]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += v[p][e] * v[p][e];
        }
    }
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
    __syncthreads();
    const float inv = rms_scale(block_total(red, T >> 6), 1.0f / (float)m, eps);
#pragma unroll
    for (int p = 0; p < kFuseNormPasses; ++p) {
        const int c = (p * T + tid) * 8;
        if (c < m) {
            float wv[8], o[8];
            unpack8h(*(const u32x4_t *)(norm_w + c), wv);
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = v[p][e] * inv * wv[e];
            *(u32x4_t *)(xn + base + c) = pack8h(o);
        }
    }
}

// Plain fp16 epilogue of the QKV matmul + rotary embedding of the q and k heads + append of k (rotated) and v to the
// cache at each row's position.  grid (row, slice of the heads); a thread owns eight consecutive rotation pairs of one
// head, or eight v elements.  q goes to its place in qkv (the attention kernel reads it there), k and v to the cache only.
__global__ __launch_bounds__(256) void skinny_finish_rope_kernel(const float *__restrict__ partial, int splits, int n, int m,
                                                                 uint16_t *__restrict__ qkv, uint16_t *__restrict__ kc, uint16_t *__restrict__ vc,
                                                                 const float *__restrict__ rope, int h, int g, int d, int cap, SeqTable st)
{
    const int i = blockIdx.x;
    const RowInfo ri = row_info(st, i);
    const int hd2 = d >> 1, per_head = hd2 >> 3;
    const size_t base = (size_t)i * m, split_stride = (size_t)n * m;
    const size_t tok = ((size_t)ri.slot * cap + ri.pos) * (size_t)(g * d);
    const int items = (h + g) * per_head;
    for (int u = blockIdx.y * 256 + threadIdx.x; u < items; u += gridDim.y * 256) {
        const int j = u / per_head, t0 = (u - j * per_head) * 8;
        float a[8], b[8];
        sum_splits8(partial, splits, split_stride, base + j * d + t0, a);
        sum_splits8(partial, splits, split_stride, base + j * d + t0 + hd2, b);
        unpack8h(pack8h(a), a);                            // the fp16 rounding of the plain epilogue comes first
        unpack8h(pack8h(b), b);
        const float *cs = rope + ((size_t)ri.pos * hd2 + t0) * 2;
        float oa[8], ob[8];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            const float4_t c2 = *(const float4_t *)(cs + e * 2);          // cos, sin of t0 + e and t0 + e + 1
            oa[e] = a[e] * c2.x - b[e] * c2.y, oa[e + 1] = a[e + 1] * c2.z - b[e + 1] * c2.w;
            ob[e] = a[e] * c2.y + b[e] * c2.x, ob[e + 1] = a[e + 1] * c2.w + b[e + 1] * c2.z;
        }
        const u32x4_t va = pack8h(oa), vb = pack8h(ob);
        if (j < h) {
            *(u32x4_t *)(qkv + base + j * d + t0) = va;
            *(u32x4_t *)(qkv + base + j * d + t0 + hd2) = vb;
        } else {
            *(u32x4_t *)(kc + tok + (size_t)(j - h) * d + t0) = va;
            *(u32x4_t *)(kc + tok + (size_t)(j - h) * d + t0 + hd2) = vb;
        }
    }
    for (int e = (blockIdx.y * 256 + threadIdx.x) * 8; e < g * d; e += gridDim.y * 256 * 8) {
        float v[8];
        sum_splits8(partial, splits, split_stride, base + (size_t)(h + g) * d + e, v);
        *(u32x4_t *)(vc + tok + e) = pack8h(v);
    }
}

struct SkinnyPlan {
    int tiles_m, splits, rounds_per_split;
};

// Split count: about one workgroup per CU when the row tiles alone do not give that many, no k range shorter than 4 rounds (unless k itself is),
// none longer than kMaxRounds; with 128-wide rounds every task has an even number of them (its scales come in packets of 256 columns).
SkinnyPlan skinny_plan(int m, int k, int kr)
{
    SkinnyPlan p;
    p.tiles_m = (m + kRowsPerBlock - 1) / kRowsPerBlock;
    const int rounds = k / kr;
    int splits = 256 / p.tiles_m;                         // about one workgroup per CU: more of them in flight measured slower (7B and 70B shapes, 16 and 64 rows)
    const int max_splits = rounds >= 4 ? rounds / 4 : 1, min_splits = (rounds + kMaxRounds - 1) / kMaxRounds;
    splits = splits > max_splits ? max_splits : splits;
    splits = splits < min_splits ? min_splits : splits;
    p.rounds_per_split = (rounds + splits - 1) / splits;
    if (kr == 128) p.rounds_per_split = (p.rounds_per_split + 1) & ~1;
    p.splits = (rounds + p.rounds_per_split - 1) / p.rounds_per_split;
    return p;
}

inline int skinny_round(int n) { return n <= 64 ? 256 : 128; }   // wider x tiles take narrower rounds: the x chunk has to fit LDS twice

template <int NF, int XR, int KR>
hipError_t launch_skinny(const SkinnyArgs &a, dim3 grid, hipStream_t stream)
{
    const size_t lds = (size_t)2 * XR * (KR + 8) * sizeof(uint16_t) + (size_t)kRowsPerBlock * (a.rounds_per_split * KR / 256 * 8 + 8) * sizeof(uint16_t);
    static std::atomic<bool> attr_done{false};   // setting the attribute twice is harmless; the flag only has to be a defined read
    if (!attr_done.load()) {
        if (hipFuncSetAttribute((const void *)skinny_q4_kernel<NF, XR, KR>, hipFuncAttributeMaxDynamicSharedMemorySize, 112 * 1024) != hipSuccess)
            return hipErrorInvalidValue;
        attr_done.store(true);
    }
    hipLaunchKernelGGL((skinny_q4_kernel<NF, XR, KR>), grid, dim3(256), lds, stream, a);
    return hipGetLastError();
}

}  // namespace

bool gemm_skinny_eligible(const relax_qmat &w, const void *x, int n, int epi)
{
    if (n < 1 || n > kSkinnyMaxN) return false;
    if (w.k % kRound != 0) return false;
    if (gshift_of(w.group) < 0) return false;
    if ((reinterpret_cast<uintptr_t>(w.q) & 15) != 0 || (reinterpret_cast<uintptr_t>(w.s) & 15) != 0) return false;
    if ((reinterpret_cast<uintptr_t>(x) & 15) != 0) return false;
    return epi == EPI_SWIGLU ? w.m % 8 == 0 : w.m % 4 == 0;
}

// fp32 elements of workspace the partial tiles of one matmul need
size_t gemm_skinny_partial_floats(int m, int k, int n)
{
    if (k % kRound != 0) return 0;
    size_t worst = 0;                                     // n rows may run with either round size: take the larger plan
    for (int kr : {256, 128}) {
        const size_t v = (size_t)skinny_plan(m, k, kr).splits * (size_t)n * (size_t)m;
        worst = v > worst ? v : worst;
    }
    return worst;
}

bool gemm_skinny_fuse_ok(const relax_qmat &w, int epi, const SkinnyFuse &f)
{
    if (epi == EPI_RESID_F32 || epi == EPI_RESID_F16)
        return f.norm_w && f.xn && w.m % 8 == 0 && w.m <= kFuseNormPasses * 2048 &&
               ((reinterpret_cast<uintptr_t>(f.norm_w) | reinterpret_cast<uintptr_t>(f.xn)) & 15) == 0;
    if (epi == EPI_F16)
        return f.dm && f.cache && f.st && f.dm->head_dim % 16 == 0 && w.m == (f.dm->n_heads + 2 * f.dm->n_kv_heads) * f.dm->head_dim &&
               ((reinterpret_cast<uintptr_t>(f.cache->k) | reinterpret_cast<uintptr_t>(f.cache->v) | reinterpret_cast<uintptr_t>(f.cache->rope)) & 15) == 0;
    return false;
}

hipError_t launch_gemm_skinny(const uint16_t *x, const relax_qmat &w, int n, int epi, uint16_t *out_f16, float *out_f32, const void *resid,
                              float *partial, hipStream_t stream, const SkinnyFuse *fuse)
{
    const SkinnyPlan pl = skinny_plan(w.m, w.k, skinny_round(n));
    SkinnyArgs a;
    a.x = x, a.q = w.q, a.s = w.s, a.gshift = gshift_of(w.group), a.partial = partial, a.n = n, a.m = w.m, a.k = w.k, a.rounds_per_split = pl.rounds_per_split;
    dim3 grid(pl.tiles_m, pl.splits);
    hipError_t e;
    const int splits = pl.splits;
    if (n <= 16) e = launch_skinny<1, 16, 256>(a, grid, stream);
    else if (n <= 32) e = launch_skinny<1, 32, 256>(a, grid, stream);
    else if (n <= 64) e = launch_skinny<2, 64, 256>(a, grid, stream);
    else e = launch_skinny<4, 128, 128>(a, grid, stream);
    if (e != hipSuccess) return e;
    return launch_skinny_finish(partial, splits, n, w.m, epi, out_f16, out_f32, resid, stream, fuse);
}

// The finishing pass alone: out = epilogue(sum over splits, in order, of partial[s][i][r]) (+ the folded light step).  Also serves the
// k-split form of the tiled GEMM, whose partial tiles have the same layout.
hipError_t launch_skinny_finish(const float *partial, int splits, int n, int m, int epi, uint16_t *out_f16, float *out_f32, const void *resid,
                                hipStream_t stream, const SkinnyFuse *fuse)
{
    struct { int m; } w = {m};
    if (fuse) {                                           // the caller checked gemm_skinny_fuse_ok
        if (epi == EPI_RESID_F32)
            hipLaunchKernelGGL(skinny_finish_norm_kernel<EPI_RESID_F32>, dim3(n), dim3(norm_block_threads(w.m, n)), 0, stream, partial, splits, n, w.m, out_f16, out_f32, resid,
                               fuse->norm_w, fuse->xn, fuse->eps);
        else if (epi == EPI_RESID_F16)
            hipLaunchKernelGGL(skinny_finish_norm_kernel<EPI_RESID_F16>, dim3(n), dim3(norm_block_threads(w.m, n)), 0, stream, partial, splits, n, w.m, out_f16, out_f32, resid,
                               fuse->norm_w, fuse->xn, fuse->eps);
        else if (epi == EPI_F16) {
            const relax_layer_dims &dm = *fuse->dm;
            const int items = (dm.n_heads + dm.n_kv_heads) * (dm.head_dim / 16);
            hipLaunchKernelGGL(skinny_finish_rope_kernel, dim3(n, (items + 255) / 256), dim3(256), 0, stream, partial, splits, n, w.m, out_f16, fuse->cache->k,
                               fuse->cache->v, fuse->cache->rope, dm.n_heads, dm.n_kv_heads, dm.head_dim, dm.kv_capacity, *fuse->st);
        }
        else return hipErrorInvalidValue;
        return hipGetLastError();
    }
    const int width = epi == EPI_SWIGLU ? w.m / 2 : w.m;
    const unsigned fb = (unsigned)(((size_t)n * width / 4 + 255) / 256);
    switch (epi) {
    case EPI_F16: hipLaunchKernelGGL(skinny_finish_kernel<EPI_F16>, dim3(fb), dim3(256), 0, stream, partial, splits, n, w.m, out_f16, out_f32, resid); break;
    case EPI_RESID_F32: hipLaunchKernelGGL(skinny_finish_kernel<EPI_RESID_F32>, dim3(fb), dim3(256), 0, stream, partial, splits, n, w.m, out_f16, out_f32, resid); break;
    case EPI_RESID_F16: hipLaunchKernelGGL(skinny_finish_kernel<EPI_RESID_F16>, dim3(fb), dim3(256), 0, stream, partial, splits, n, w.m, out_f16, out_f32, resid); break;
    case EPI_SWIGLU: hipLaunchKernelGGL(skinny_finish_kernel<EPI_SWIGLU>, dim3(fb), dim3(256), 0, stream, partial, splits, n, w.m, out_f16, out_f32, resid); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace relax
