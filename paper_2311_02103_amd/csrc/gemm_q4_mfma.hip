// Fused int4-decode GEMM for large n (prefill): out[i,r] = sum_c x[i,c] * (u(r,c) - 8) * s[r, c/32].
//
// At large n the contraction is dense and MFMA-bound (Relax, Sec. 5.1: library-grade GEMM for batch sizes
// other than 1; Sec. 4.2: the 4-bit decode stays fused into the matmul).  Mapping for gfx950:
//   - v_mfma_f32_32x32x16_f16, fp32 accumulate.  The 256 x 256 tile (weight rows x x-rows) runs as eight wavefronts,
//     two per SIMD with up to 256 registers each (64 x 128 outputs per wavefront), so that one wavefront's decode, LDS
//     traffic and waits run under the other's MFMAs; the narrower tiles and the fp16-weight variant run as four
//     wavefronts (2 x 2), one per SIMD (128 x 256 as eight wavefronts of 64 x 64 was measured 4 to 11 % slower than as
//     four of 64 x 128: twice the fragment reads per MFMA).
//   - Both operands go through LDS in 64-wide k blocks, double buffered with ONE LDS-only barrier per block
//     (global loads of the next block stay in flight across it).  The packed weights are decoded on the way in,
//     once per workgroup: every thread loads its share of the codes and the group scale of one weight row, turns
//     them into fp16 values and writes them to LDS.  Decode = merge the nibbles into the mantissa of fp16
//     1024.0, remove the offset exactly (1024+u-1032, (1024+16u)/16-72), multiply by the group scale: 13
//     packed-fp16 VALU ops per 8 weights.  A quarter of a block's loads, decode and LDS writes is placed next to the
//     MFMAs of each of its four k steps.
//   - What bounds it: with realistic operand values the matrix pipes of this chip run well below the rate they reach on
//     all-zero operands (the vendor's fp16 GEMM: 1.5 against 2.3 PFLOP/s at 8192^3; 0.86 to 1.19 PFLOP/s on the four
//     shapes of the 7B layer at n = 2048), so timing a variant on dummy LDS contents says nothing about its staging cost.
//   - Each 8-wide k packet is kept in LDS in the order [e0 e4 e1 e5 e2 e6 e3 e7] -- the nibble pairs the decode
//     produces; the x tile is permuted the same way when it is staged.  The order of k inside an MFMA is free
//     as long as A and B agree.  Rows are padded to 144 bytes: 16-byte reads and writes of consecutive rows hit
//     distinct banks.
//   - For the gate/up matrix a workgroup tile is 128 gate rows + the 128 matching up rows and a wavefront owns
//     matching fragments of both, so SwiGLU is an element-wise epilogue on the accumulators.
//   - n, m need not be multiples of the tile: rows are clamped on load and masked on store (one binary for
//     every n: 17, 511, 2048 ...).  k must be a multiple of 128 (else the matvec path serves the call).
//     Narrower tiles (64 weight rows per wavefront; 32 or 64 x-rows per wavefront) are picked by the launcher
//     when the wide one would leave CUs idle.
#include <atomic>

#include "relax_common.h"

namespace relax {

namespace {

std::atomic<int> g_waves_per_simd{2};

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int BK = 64;                  // k per main-loop step
constexpr int kPitch = BK + 8;          // LDS row pitch in halfs (144 bytes)

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

// (w & mask) | bits as one VALU op (mask from a scalar register, bits from a vector register: the encoding
// takes no literal and only one scalar source)
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t bits)
{
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(bits));
    return r;
}

// one packed word (8 codes, elements 0..7) and its group scale (fp16 pair s,s) -> 8 fp16 weights in the packet
// order [e0 e4 e1 e5 e2 e6 e3 e7]; every step is exact except the final multiply by the scale
__device__ __forceinline__ half8_t decode_word(uint32_t w, uint32_t s2)
{
    const uint32_t w8 = w >> 8;
    const uint32_t a0 = and_or(w, 0x000F000Fu, 0x64006400u);   // 1024 + u   : e0, e4
    const uint32_t a1 = and_or(w, 0x00F000F0u, 0x64006400u);   // 1024 + 16u : e1, e5
    const uint32_t a2 = and_or(w8, 0x000F000Fu, 0x64006400u);  // e2, e6
    const uint32_t a3 = and_or(w8, 0x00F000F0u, 0x64006400u);  // e3, e7
    const uint32_t kNeg1032 = 0xE408E408u, kSixteenth = 0x2C002C00u, kNeg72 = 0xD480D480u;
    uint4 r;
    r.x = pk_mul(pk_add(a0, kNeg1032), s2);
    r.y = pk_mul(pk_fma(a1, kSixteenth, kNeg72), s2);
    r.z = pk_mul(pk_add(a2, kNeg1032), s2);
    r.w = pk_mul(pk_fma(a3, kSixteenth, kNeg72), s2);
    return __builtin_bit_cast(half8_t, r);
}

// 3-bit weights in the native word layout (three words per group of 32 columns: word w, position j holds column 2(5w+j)
// in bits 3j.. and column 2(5w+j)+1 in bits 16+3j..; bit i of columns 30 / 31 is bit 15 / 31 of word i): the four fp16 pairs
// of packet t (columns 8t .. 8t+7 of the group, NATURAL order) times the group scale.  v_and_or_b32 merges a pair of codes
// into the mantissas of fp16 (1024, 1024) at weight 1, 8 or 64; one packed fma removes offset and weight exactly
// ((1024 + f u) / f - (1024 / f + 4) = u - 4), one packed multiply applies the scale.
__device__ __forceinline__ half8_t decode_q3_packet(uint32_t w0, uint32_t w1, uint32_t w2, int t, uint32_t s2)
{
    const uint32_t base = 0x64006400u;
    const uint32_t kOne = 0x3C003C00u, kEighth = 0x30003000u, k64th = 0x24002400u;          // 1, 1/8, 1/64
    const uint32_t kNeg1028 = 0xE404E404u, kNeg132 = 0xD820D820u, kNeg20 = 0xCD00CD00u;     // -(1024 / f + 4)
    uint32_t r[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int p = 4 * t + q;                              // pair p = columns 2p, 2p + 1
        uint32_t pair;
        int cls;                                              // 0: weight 1, 1: weight 8, 2: weight 64
        if (p == 15) {
            uint32_t g = and_or(w0 >> 15, 0x00010001u, base);
            g = and_or(w1 >> 14, 0x00020002u, g);
            pair = and_or(w2 >> 13, 0x00040004u, g), cls = 0;
        } else {
            const uint32_t w = p / 5 == 0 ? w0 : p / 5 == 1 ? w1 : w2;
            const int j = p % 5;
            const uint32_t v = j >= 3 ? w >> 9 : w;
            cls = j >= 3 ? j - 3 : j;
            pair = and_or(v, cls == 0 ? 0x00070007u : cls == 1 ? 0x00380038u : 0x01C001C0u, base);
        }
        const uint32_t scaled = cls == 0 ? pk_fma(pair, kOne, kNeg1028) : cls == 1 ? pk_fma(pair, kEighth, kNeg132) : pk_fma(pair, k64th, kNeg20);
        r[q] = pk_mul(scaled, s2);
    }
    uint4 o = {r[0], r[1], r[2], r[3]};
    return __builtin_bit_cast(half8_t, o);
}

struct GemmArgs {
    const uint16_t *x;       // [n,k] fp16
    const uint32_t *q;       // [m,k/8]; Q3 kernels: [m, 3 k / 32] words of the native 3-bit layout
    const uint16_t *s;       // [m, k / (32 << gshift)]
    int32_t gshift;          // 32-column sub-group index >> gshift = scale index (quantisation group 32, 64 or 128)
    const uint16_t *wh;      // FP16W kernels: plain fp16 weights [m,k] instead of q, s
    int32_t n, m, k;
    int32_t ldm;             // row pitch of out / resid in elements; 0: m (a launch on a range of the weight rows brings the matrix's m here)
    int32_t epi;
    int32_t tiles_m;         // weight-row tiles of the launch (the grid is one-dimensional: tiles_m * x-row tiles * k splits)
    int32_t tiles_n;         // x-row tiles
    int32_t kb_per_split;    // k blocks (of BK columns) per k split, even; one split: all of them
    float *partial;          // more than one k split: [split][n][m] fp32 partial tiles, finished by the few-row kernel's finishing pass
    uint16_t *out_f16;       // EPI_F16: [n,m]; EPI_RESID_F16: [n,m]; EPI_SWIGLU: [n,m/2]
    float *out_f32;          // EPI_RESID_F32: [n,m]
    const void *resid;       // EPI_RESID_F32: fp16 [n,m]; EPI_RESID_F16: fp32 [n,m]
};

// One-dimensional grid of tiles_m * (x-row tiles) workgroups.  Wavefront w owns MF fragments of 32 weight rows (w & 1 picks which)
// and NF fragments of 32 x-rows (w >> 1 picks which) of the workgroup tile of 64 MF weight rows x 64 NF x-rows.
// LDS row r of the weight tile is weight row m0 + r, except for EPI_SWIGLU: rows [0, 32 MF) are gate rows
// g0 + r and rows [32 MF, 64 MF) the up rows F + g0 + (r - 32 MF).
// FP16W: the weights are plain fp16 (the fp16-weight configurations of the paper's LLM charts, Sec. 5.1): the staging copies
// 16-byte packets instead of decoding words, everything else is the same kernel.
// WM x WN: wavefronts along the weight rows and along the x rows.  2 x 2: four wavefronts, one per SIMD, each with up to 512
// registers.  4 x 2: eight wavefronts, two per SIMD with up to 256 registers each, so that one wavefront's decode, LDS
// traffic and waits run under the other's MFMAs (with one wavefront per SIMD the matrix pipe was busy 37 % of the time:
// counters in profiles/).
// Q3: 3-bit weights in the native word layout (Sec. 5.3 of the paper deploys 3-bit models): a thread stages whole groups of 32
// columns (three words), the decode yields the columns in natural order, so the x tile is staged unpermuted.
template <int EPI, int MF, int NF, bool FP16W = false, int WM = 2, int WN = 2, bool Q3 = false>
__global__ __launch_bounds__(WM * WN * 64) void gemm_q4_mfma_kernel(GemmArgs a)
{
    static_assert(!(FP16W && Q3), "one weight format per kernel");
    constexpr int ST = 2;                                 // register stages; four were measured and gained nothing
    constexpr int kThreadsG = WM * WN * 64;
    constexpr int BM = 32 * MF * WM, BN = 32 * NF * WN;
    // packed words a thread decodes per k block: its share of the BM x 8 words of the weight tile (2, 4 or 8: every thread
    // stages weights, so the staging has no branch for the compiler's wait-count pass to merge across)
    constexpr int W = BM * 8 / kThreadsG;
    constexpr int TPR = 8 / W;                            // threads per weight row
    constexpr int XP = BN * 8 / kThreadsG;                // 16-byte x packets a thread stages per k block
    static_assert((W == 2 || W == 4 || W == 8) && XP >= 1, "staging roles");
    static_assert(!Q3 || W >= 4, "a thread stages whole 3-bit groups");
    constexpr int WV = W < 4 ? 1 : W / 4;                 // 16-byte (W = 2: 8-byte) loads of packed words per thread and k block
    constexpr int kABuf = BM * kPitch, kBBuf = BN * kPitch;
    extern __shared__ __align__(16) uint16_t lds[];       // A[2][BM][kPitch], B[2][BN][kPitch]
    uint16_t *const As = lds, *const Bs = lds + 2 * kABuf;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row32 = lane & 31, hf = lane >> 5;
    const int wm = wave % WM, wn = wave / WM;
    // Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own L2.  Renumber them so
    // that an XCD owns a contiguous run of tiles: the x tiles a workgroup streams are then fetched into one L2 instead of eight.
    const int nb = gridDim.x, xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    const int tile = xcd * (nb >> 3) + min(xcd, nb & 7) + idx;
    // Inside an XCD's run the x-row tile changes fastest within a PAIR of x-row tiles: a round of 32 workgroups then is 16
    // weight-row tiles x 2 x-row tiles, and an XCD streams half of the weight matrix instead of all of it (requests of the L2s
    // to the fabric on the 7B gate/up shape at n = 2048: 304 MB against 456 MB; neither operand fits a 4 MB L2).
    const int per_split = a.tiles_m * a.tiles_n, split = tile / per_split, t2 = tile - split * per_split;
    const int pair = t2 / (2 * a.tiles_m), r2 = t2 - pair * 2 * a.tiles_m;
    const bool whole = 2 * pair + 1 < a.tiles_n;          // the last pair of an odd count is a single tile
    const int tile_m = whole ? r2 >> 1 : r2, tile_n = whole ? 2 * pair + (r2 & 1) : 2 * pair;
    const int n0 = tile_n * BN;
    const int kw = a.k >> 3;
    const int F = a.m >> 1;
    const int ldm = a.ldm > 0 ? a.ldm : a.m;

    // ---- staging roles ----
    const int arow = tid / TPR, aword0 = (tid % TPR) * W;
    int grow;
    if (EPI == EPI_SWIGLU) {
        const int g0 = tile_m * (BM / 2);
        grow = arow < BM / 2 ? min(g0 + arow, F - 1) : F + min(g0 + arow - BM / 2, F - 1);
    } else {
        grow = min(tile_m * BM + arow, a.m - 1);
    }
    const uint32_t *qsrc = FP16W ? nullptr : Q3 ? a.q + ((size_t)grow * (a.k >> 5) + (aword0 >> 2)) * 3 : a.q + (size_t)grow * kw + aword0;
    const uint16_t *ssrc = FP16W ? nullptr : a.s + (size_t)grow * scales_per_row(a.k, a.gshift);
    const int sub0 = aword0 >> 2;                         // first 32-column sub-group of this thread's words inside a k block
    const uint16_t *hsrc = FP16W ? a.wh + (size_t)grow * a.k + aword0 * 8 : nullptr;
    const uint16_t *xsrc[XP];
#pragma unroll
    for (int p = 0; p < XP; ++p) {
        const int pk = tid + p * kThreadsG;
        xsrc[p] = a.x + (size_t)min(n0 + (pk >> 3), a.n - 1) * a.k + (pk & 7) * 8;
    }

    // Staged registers of one k block: packed codes + scales of this thread's weight row part, and its x packets.
    struct Stage {
        uint4 wq[FP16W ? W : WV];                         // packed words (W = 2: in .x, .y), or one 16-byte packet of fp16 weights per word
        uint32_t wsc;
        uint4 xr[XP];
    };
    const int kb0 = split * a.kb_per_split;               // this workgroup's k range: blocks kb0 .. kb0 + nkb - 1
    const int nkb = min(a.kb_per_split, a.k / BK - kb0);
    // The loads of k block kb, in four shares: share `part` is issued next to k step `part` of the running block -- a
    // workgroup that issued all its loads in one burst at the top of a block filled the address queue of the texture unit and
    // stalled in front of its own MFMAs.  Loads return in order, so the order of issue is what the wait counts stand on:
    // weights first (the decode of share 0 needs them first), then per share the x packets.
    auto stage_load = [&](Stage &S, int kb, int part) {   // kb is clamped: the tail re-reads the last block (never consumed)
        kb = kb0 + min(kb, nkb - 1);
        if (FP16W) {
#pragma unroll
            for (int i = 0; i < W; ++i)
                if (i * 4 / W == part) S.wq[i] = *(const uint4 *)(hsrc + kb * BK + i * 8);
        } else {
#pragma unroll
            for (int i = 0; i < WV; ++i) {
                if (i * 2 != part) continue;
                if (Q3) {                                 // group i of this thread: three words, 4-byte aligned
                    const uint32_t *g3 = qsrc + (kb * (BK / 32) + i) * 3;
                    S.wq[i].x = g3[0], S.wq[i].y = g3[1], S.wq[i].z = g3[2];
                } else if (W == 2) {
                    const uint2 two = *(const uint2 *)(qsrc + kb * (BK / 8));
                    S.wq[0].x = two.x, S.wq[0].y = two.y;
                } else {
                    S.wq[i] = *(const uint4 *)(qsrc + kb * (BK / 8) + i * 4);
                }
            }
            if (part == 1) {
                // scale of sub-group g: ssrc[g >> gshift] (neighbouring sub-groups share it when the group is wider than 32)
                const int g = kb * (BK / 32) + sub0;
                if (W == 8) S.wsc = (uint32_t)ssrc[g >> a.gshift] | ((uint32_t)ssrc[(g + 1) >> a.gshift] << 16);
                else S.wsc = ssrc[g >> a.gshift];
            }
        }
#pragma unroll
        for (int p = 0; p < XP; ++p)
            if (p * 4 / XP == part) S.xr[p] = *(const uint4 *)(xsrc[p] + kb * BK);
    };
    // a whole block's loads in the order the running loop issues them (prologue): the compiler's wait counts at the loop
    // head are the merge of this order and the loop's own, so the two must agree or every wait in the loop is pessimistic
    auto stage_load_all = [&](Stage &S, int kb) {
#pragma unroll
        for (int part = 0; part < 4; ++part) {
            stage_load(S, kb, part);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // quarter `part` (0..3) of the decode + LDS write of a staged block
    auto stage_store = [&](const Stage &S, int buf, int part) {
        uint16_t *ad = As + buf * kABuf + arow * kPitch + aword0 * 8;
#pragma unroll
        for (int i = 0; i < W; ++i) {
            if (i * 4 / W != part) continue;
            if (FP16W) {                                  // same packet order as the decode and the x tile
                const uint4 &h = S.wq[FP16W ? i : 0];
                uint4 o;
                o.x = __builtin_amdgcn_perm(h.z, h.x, 0x05040100u);
                o.y = __builtin_amdgcn_perm(h.z, h.x, 0x07060302u);
                o.z = __builtin_amdgcn_perm(h.w, h.y, 0x05040100u);
                o.w = __builtin_amdgcn_perm(h.w, h.y, 0x07060302u);
                *(uint4 *)(ad + i * 8) = o;
                continue;
            }
            const uint4 &wv = S.wq[i >> 2];
            const uint32_t word = (i & 3) == 0 ? wv.x : (i & 3) == 1 ? wv.y : (i & 3) == 2 ? wv.z : wv.w;
            const uint32_t sc = (W == 8 && i >= 4) ? (S.wsc >> 16) : (S.wsc & 0xFFFFu);
            if (Q3) *(half8_t *)(ad + i * 8) = decode_q3_packet(wv.x, wv.y, wv.z, i & 3, sc | (sc << 16));
            else *(half8_t *)(ad + i * 8) = decode_word(word, sc | (sc << 16));
        }
        uint16_t *bd = Bs + buf * kBBuf;
#pragma unroll
        for (int p = 0; p < XP; ++p) {
            if (p * 4 / XP != part) continue;
            const int pk = tid + p * kThreadsG;
            // [x0 x1 | x2 x3 | x4 x5 | x6 x7] -> [x0 x4 | x1 x5 | x2 x6 | x3 x7]
            uint4 o = S.xr[p];                            // Q3: the decode yields natural order
            if (!Q3) {
                o.x = __builtin_amdgcn_perm(S.xr[p].z, S.xr[p].x, 0x05040100u);
                o.y = __builtin_amdgcn_perm(S.xr[p].z, S.xr[p].x, 0x07060302u);
                o.z = __builtin_amdgcn_perm(S.xr[p].w, S.xr[p].y, 0x05040100u);
                o.w = __builtin_amdgcn_perm(S.xr[p].w, S.xr[p].y, 0x07060302u);
            }
            *(uint4 *)(bd + (pk >> 3) * kPitch + (pk & 7) * 8) = o;
        }
    };
    // LDS-only workgroup barrier: the global loads of later k blocks stay in flight across it
    auto lds_barrier = [&]() {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
    };

    // ---- MFMA roles ----
    int afrag_off[MF];                                    // offset of this lane's fragment rows inside a weight tile
#pragma unroll
    for (int f = 0; f < MF; ++f) {
        int rb;
        if (EPI == EPI_SWIGLU) rb = (f / (MF / 2)) * (BM / 2) + (wm * (MF / 2) + f % (MF / 2)) * 32;
        else rb = (wm * MF + f) * 32;
        afrag_off[f] = (rb + row32) * kPitch + hf * 8;
    }
    const int bfrag_off = (wn * NF * 32 + row32) * kPitch + hf * 8;

    float16_t acc[MF][NF];
#pragma unroll
    for (int f = 0; f < MF; ++f)
#pragma unroll
        for (int j = 0; j < NF; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[f][j][v] = 0.0f;

    // One k block: MFMAs on LDS buffer `buf` while the staged block S is decoded into the other buffer.  The
    // fragments of k step ks+1 are requested before the MFMAs of step ks are issued, and a quarter of the decode
    // is placed next to each step's MFMAs; the scheduling fences keep the compiler from undoing either.
    auto block = [&](int buf, const Stage &S, Stage &L, int kb_load) {
        const uint16_t *ab = As + buf * kABuf, *bb = Bs + buf * kBBuf + bfrag_off;
        half8_t af[2][MF], bf[2][NF];
#pragma unroll
        for (int f = 0; f < MF; ++f) af[0][f] = *(const half8_t *)(ab + afrag_off[f]);
#pragma unroll
        for (int j = 0; j < NF; ++j) bf[0][j] = *(const half8_t *)(bb + j * 32 * kPitch);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks + 1 < BK / 16) {
#pragma unroll
                for (int f = 0; f < MF; ++f) af[nxt][f] = *(const half8_t *)(ab + afrag_off[f] + (ks + 1) * 16);
#pragma unroll
                for (int j = 0; j < NF; ++j) bf[nxt][j] = *(const half8_t *)(bb + j * 32 * kPitch + (ks + 1) * 16);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (WM * WN > 4) __builtin_amdgcn_s_setprio(1);      // two wavefronts per SIMD: the one that has its fragments issues its MFMAs first
#pragma unroll
            for (int j = 0; j < NF; ++j)
#pragma unroll
                for (int f = 0; f < MF; ++f)
                    acc[f][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[cur][f], bf[cur][j], acc[f][j], 0, 0, 0);
            if (WM * WN > 4) __builtin_amdgcn_s_setprio(0);
            stage_load(L, kb_load, ks);
            stage_store(S, buf ^ 1, ks);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Software pipeline over k blocks, ST register stages deep: the global loads of block kb+ST are issued during block kb
    // (a share next to each k step) into the stage whose block was decoded during block kb-1, and are consumed (decoded
    // into LDS) during block kb+ST-1, ST-1 blocks of MFMAs later (the k blocks of a workgroup are a multiple of ST).
    Stage S[ST];
    stage_load_all(S[0], 0);
#pragma unroll
    for (int part = 0; part < 4; ++part) stage_store(S[0], 0, part);
    lds_barrier();
#pragma unroll
    for (int d = 1; d < ST; ++d) stage_load_all(S[d], d);
    for (int kb = 0; kb < nkb; kb += ST) {
#pragma unroll
        for (int b = 0; b < ST; ++b) {
            // MFMAs on buffer b & 1 (block kb+b), block kb+b+1 decoded into the other buffer, loads of block kb+b+ST
            block(b & 1, S[(b + 1) % ST], S[b], kb + b + ST);
            lds_barrier();
        }
    }

    // ---- epilogue.  acc[f][j][v]: tile row of fragment f + 8 (v/4) + 4 (lane/32) + v%4, x row n0 + 32 (NF wn + j) + lane%32 ----
    if (a.partial) {
        // k split: the raw fp32 tile goes to partial[split][x row][weight row] (gate rows first, up rows from F on, as in the
        // matrix), and the finishing pass adds the splits in order and applies the epilogue
#pragma unroll
        for (int j = 0; j < NF; ++j) {
            const int xrow = n0 + (wn * NF + j) * 32 + row32;
            if (xrow >= a.n) continue;
            float *dst = a.partial + ((size_t)split * a.n + xrow) * a.m;
#pragma unroll
            for (int f = 0; f < MF; ++f)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int off = b * 8 + hf * 4;
                    int row;                                     // matrix row of this granule of four
                    bool ok;
                    if (EPI == EPI_SWIGLU) {
                        const int g = tile_m * (BM / 2) + (wm * (MF / 2) + f % (MF / 2)) * 32 + off;
                        row = (f / (MF / 2)) * F + g, ok = g < F;
                    } else {
                        row = tile_m * BM + (wm * MF + f) * 32 + off, ok = row < a.m;
                    }
                    if (ok)
                        *(float4 *)(dst + row) = make_float4(acc[f][j][b * 4], acc[f][j][b * 4 + 1], acc[f][j][b * 4 + 2], acc[f][j][b * 4 + 3]);
                }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < NF; ++j) {
        const int xrow = n0 + (wn * NF + j) * 32 + row32;
        if (xrow >= a.n) continue;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int off = b * 8 + hf * 4;
            if (EPI == EPI_SWIGLU) {
#pragma unroll
                for (int f = 0; f < MF / 2; ++f) {
                    const int g = tile_m * (BM / 2) + (wm * (MF / 2) + f) * 32 + off;
                    if (g < F) {                                 // F % 4 == 0 is checked by the launcher
                        uint16_t o[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float gte = acc[f][j][b * 4 + r], up = acc[f + MF / 2][j][b * 4 + r];
                            o[r] = f2h(gte / (1.0f + __expf(-gte)) * up);
                        }
                        *(uint2 *)(a.out_f16 + (size_t)xrow * F + g) = make_uint2(o[0] | ((uint32_t)o[1] << 16), o[2] | ((uint32_t)o[3] << 16));
                    }
                }
            } else {
#pragma unroll
                for (int f = 0; f < MF; ++f) {
                    const int r0 = tile_m * BM + (wm * MF + f) * 32 + off;
                    if (r0 < a.m) {                              // m % 4 == 0 is checked by the launcher
                        const size_t at = (size_t)xrow * ldm + r0;
                        float v[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = acc[f][j][b * 4 + r];
                        if (EPI == EPI_RESID_F32) {
                            const uint2 xx = *(const uint2 *)((const uint16_t *)a.resid + at);
                            float4 o;
                            o.x = h2f((uint16_t)(xx.x & 0xFFFFu)) + v[0], o.y = h2f((uint16_t)(xx.x >> 16)) + v[1];
                            o.z = h2f((uint16_t)(xx.y & 0xFFFFu)) + v[2], o.w = h2f((uint16_t)(xx.y >> 16)) + v[3];
                            *(float4 *)(a.out_f32 + at) = o;
                        } else {
                            if (EPI == EPI_RESID_F16) {
                                const float4 rr = *(const float4 *)((const float *)a.resid + at);
                                v[0] += rr.x, v[1] += rr.y, v[2] += rr.z, v[3] += rr.w;
                            }
                            *(uint2 *)(a.out_f16 + at) =
                                make_uint2(f2h(v[0]) | ((uint32_t)f2h(v[1]) << 16), f2h(v[2]) | ((uint32_t)f2h(v[3]) << 16));
                        }
                    }
                }
            }
        }
    }
}

template <int MF, int NF, bool FP16W = false, int WM = 2, int WN = 2, bool Q3 = false>
hipError_t launch_tile(const GemmArgs &a_in, hipStream_t stream, int splits)
{
    constexpr int BM = 32 * MF * WM, BN = 32 * NF * WN, kThreadsG = WM * WN * 64;
    const int rows = a_in.epi == EPI_SWIGLU ? a_in.m / 2 : a_in.m, per_block = a_in.epi == EPI_SWIGLU ? BM / 2 : BM;
    GemmArgs a = a_in;
    a.tiles_m = (rows + per_block - 1) / per_block;
    a.tiles_n = (a.n + BN - 1) / BN;
    const int nkb = a.k / BK, tiles = a.tiles_m * a.tiles_n;
    if (splits < 2) a.partial = nullptr, a.kb_per_split = nkb, splits = 1;
    dim3 grid(tiles * splits);
    const size_t lds = 2 * (size_t)(BM + BN) * kPitch * sizeof(uint16_t);    // up to 147456 bytes: one workgroup per CU
    static std::atomic<bool> attr_done{false};   // setting the attribute twice is harmless; the flag only has to be a defined read
    if constexpr (FP16W || Q3) {                          // plain matmuls only: one epilogue, one pass over k
        if (a.epi != EPI_F16 || splits != 1) return hipErrorInvalidValue;
        if (!attr_done.load()) {
            if (hipFuncSetAttribute((const void *)gemm_q4_mfma_kernel<EPI_F16, MF, NF, FP16W, WM, WN, Q3>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
                return hipErrorInvalidValue;
            attr_done.store(true);
        }
        hipLaunchKernelGGL((gemm_q4_mfma_kernel<EPI_F16, MF, NF, FP16W, WM, WN, Q3>), grid, dim3(kThreadsG), lds, stream, a);
        return hipGetLastError();
    }
    if (!attr_done.load()) {
        const void *ks[4] = {(const void *)gemm_q4_mfma_kernel<EPI_F16, MF, NF, false, WM, WN>, (const void *)gemm_q4_mfma_kernel<EPI_RESID_F32, MF, NF, false, WM, WN>,
                             (const void *)gemm_q4_mfma_kernel<EPI_RESID_F16, MF, NF, false, WM, WN>, (const void *)gemm_q4_mfma_kernel<EPI_SWIGLU, MF, NF, false, WM, WN>};
        for (const void *kf : ks)
            if (hipFuncSetAttribute(kf, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return hipErrorInvalidValue;
        attr_done.store(true);
    }
    switch (a.epi) {
    case EPI_F16: hipLaunchKernelGGL((gemm_q4_mfma_kernel<EPI_F16, MF, NF, false, WM, WN>), grid, dim3(kThreadsG), lds, stream, a); break;
    case EPI_RESID_F32: hipLaunchKernelGGL((gemm_q4_mfma_kernel<EPI_RESID_F32, MF, NF, false, WM, WN>), grid, dim3(kThreadsG), lds, stream, a); break;
    case EPI_RESID_F16: hipLaunchKernelGGL((gemm_q4_mfma_kernel<EPI_RESID_F16, MF, NF, false, WM, WN>), grid, dim3(kThreadsG), lds, stream, a); break;
    case EPI_SWIGLU: hipLaunchKernelGGL((gemm_q4_mfma_kernel<EPI_SWIGLU, MF, NF, false, WM, WN>), grid, dim3(kThreadsG), lds, stream, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

// Test switch ("gemm_waves_per_simd"): the 256 x 256 tile runs as eight wavefronts of 64 x 128 (2, the default) or as four of
// 128 x 128 (1).  Same arithmetic per output element in the same order either way: results are identical.
void gemm_set_waves_per_simd(int v) { g_waves_per_simd.store(v == 1 ? 1 : 2); }

// Whether the MFMA path can serve this matrix (k in whole 128-blocks, 16-byte aligned rows, 4-row store granules).
bool gemm_mfma_eligible(const relax_qmat &w, const void *x, int epi)
{
    if (w.k % (2 * BK) != 0 || gshift_of(w.group) < 0) return false;
    if ((reinterpret_cast<uintptr_t>(w.q) & 15) != 0 || (reinterpret_cast<uintptr_t>(w.s) & 1) != 0) return false;
    if ((reinterpret_cast<uintptr_t>(x) & 15) != 0) return false;
    if (epi == EPI_SWIGLU) return w.m % 8 == 0;
    return w.m % 4 == 0;
}

// Tile choice for n > 128: 256 x 256, 128 x 256 or 128 x 128 (weight rows x x-rows), whichever leaves the largest
// useful share of the rounds of workgroups over the 256 CUs (one workgroup per CU); ties go to the wider tile.
// Small n takes narrower x tiles.  A launch whose tiles would leave more than half of the CUs idle (few weight rows, few
// x rows: the output and down projections of a prefill chunk of a few hundred rows) is cut along k as well, into about one
// workgroup per CU with at least 8 k blocks each; the fp32 partial tiles go to the caller's workspace and the finishing pass
// of the few-row kernel adds them in order and applies the epilogue.
namespace {
struct TilePlan {
    int mf, nf, splits, kb_per_split;
    int m_big;               // > 0: the first m_big weight rows go through a launch of 256 x 256 tiles of their own (whole rounds of them)
};
TilePlan tile_plan(int m, int k, int n, int epi)
{
    const long rows = epi == EPI_SWIGLU ? m / 2 : m;
    const long rdiv = epi == EPI_SWIGLU ? 2 : 1;
    auto blocks = [&](int mf, int nf) { return ((rows + 64 * mf / rdiv - 1) / (64 * mf / rdiv)) * (long)((n + 64 * nf - 1) / (64 * nf)); };
    const long kCUs = 256;
    TilePlan p = {2, 1, 1, k / BK, 0};
    if (n > 128) {
        // useful share of the workgroup rounds: padding rows of ragged tiles and idle CUs of the last round both count as waste,
        // weighted by what a tile shape reaches per MFMA when the CUs are full (measured on the 7B shapes at n = 2048: the
        // 128 x 256 tile as four wavefronts reaches about nine tenths of the 256 x 256 tile as eight)
        auto score = [&](int mf, int nf, double tile_eff) {
            const long b = blocks(mf, nf);
            const double rounds = (double)((b + kCUs - 1) / kCUs);
            return tile_eff * (double)rows * (double)n / (rounds * kCUs * (64.0 * mf / rdiv) * (64.0 * nf));
        };
        const double s44 = score(4, 4, 1.0), s24 = score(2, 4, 0.9), s22 = score(2, 2, 0.6);
        if (s44 >= s24 && s44 >= s22) p.mf = 4, p.nf = 4;
        else if (s24 >= s22) p.mf = 2, p.nf = 4;
        else p.mf = 2, p.nf = 2;
        // Two launches instead of one when the 128 x 256 tile was chosen only for its rounds: whole rounds of 256 x 256
        // tiles on the first rows (the tile that reaches more per MFMA), the narrower tile on the rest.  A round of the
        // wide tile is taken as 1.6 rounds of the narrow one (129 against 80 us per round at k = 4096, n = 2048); the
        // split is made when the estimate gains a tenth (QKV of the 7B layer at n = 2048: 1.6 + 1 against 3 rounds).
        if (p.mf == 2 && p.nf == 4 && epi != EPI_SWIGLU) {
            const long tn = (n + 255) / 256;
            if (tn <= kCUs) {
                const long rows_round = (kCUs / tn) * 256;                       // weight rows of one full round of wide tiles
                const double all_small = (double)((blocks(2, 4) + kCUs - 1) / kCUs);
                double best = all_small;
                for (long r = 1; r * rows_round < rows; ++r) {
                    const long rem = rows - r * rows_round;
                    const double t = 1.6 * (double)r + (double)((((rem + 127) / 128) * tn + kCUs - 1) / kCUs);
                    if (t < best) best = t, p.m_big = (int)(r * rows_round);
                }
                if (best > 0.9 * all_small) p.m_big = 0;
            }
        }
        const long tiles = blocks(p.mf, p.nf);
        const int nkb = k / BK;
        if (n <= kSplitKMaxN && tiles <= kCUs / 2) {
            int splits = std::max(1, std::min(std::min(kSplitKMax, (int)(kCUs / tiles)), nkb / 8));
            p.kb_per_split = ((nkb + splits - 1) / splits + 1) & ~1;
            p.splits = (nkb + p.kb_per_split - 1) / p.kb_per_split;
            if (p.splits < 2) p.splits = 1, p.kb_per_split = nkb;
            if (p.splits > 1) p.m_big = 0;
        }
    } else if (n > 64) {
        p.mf = 2, p.nf = 2;
    }
    return p;
}
}  // namespace

// fp32 elements of workspace the k-split form may need for any row count up to n (0: it never splits this matrix)
size_t gemm_splitk_partial_floats(int m, int k, int n, int epi)
{
    if (k % (2 * BK) != 0) return 0;
    size_t worst = 0;
    const int top = n < kSplitKMaxN ? n : kSplitKMaxN;
    for (int nn = 256; nn <= top + 127; nn += 128) {               // splits change with the tile counts only: the top of each bracket
        const int r = nn < top ? nn : top;
        if (r <= 128) continue;
        const TilePlan p = tile_plan(m, k, r, epi);
        if (p.splits > 1) worst = std::max(worst, (size_t)p.splits * (size_t)r * (size_t)m);
    }
    return worst;
}

// k splits the launch would make for n rows with this much workspace (1: one pass over k, no finishing pass)
int gemm_mfma_splits(const relax_qmat &w, int n, int epi, const float *partial, size_t partial_floats)
{
    const TilePlan p = tile_plan(w.m, w.k, n, epi);
    if (p.splits > 1 && (!partial || (reinterpret_cast<uintptr_t>(partial) & 15) != 0 || partial_floats < (size_t)p.splits * n * w.m)) return 1;
    return p.splits;
}

// out[n,m] = x[n,k] . w[m,k]^T with plain fp16 weights: the same tiles, no decode, one pass over k
bool gemm_f16_eligible(const void *x, const void *w, const void *out, int m, int k)
{
    return k % (2 * BK) == 0 && m % 4 == 0 && ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w)) & 15) == 0 &&
           (reinterpret_cast<uintptr_t>(out) & 7) == 0;
}

hipError_t launch_gemm_f16(const uint16_t *x, const uint16_t *w, int n, int m, int k, uint16_t *out, hipStream_t stream)
{
    GemmArgs a = {};
    a.x = x, a.wh = w, a.n = n, a.m = m, a.k = k, a.epi = EPI_F16, a.out_f16 = out;
    const TilePlan p = tile_plan(m, k, n, EPI_F16);
    a.kb_per_split = k / BK;
    if (p.mf == 4) return launch_tile<4, 4, true>(a, stream, 1);    // the fp16-weight staging needs more registers than two wavefronts per SIMD leave
    if (p.nf == 4) return launch_tile<2, 4, true>(a, stream, 1);
    if (p.nf == 2) return launch_tile<2, 2, true>(a, stream, 1);
    return launch_tile<2, 1, true>(a, stream, 1);
}

// out[n,m] = x[n,k] . w[m,k]^T with 3-bit weights in the native word layout (group 32): the same tiles, one pass over k
bool gemm_q3_eligible(const void *x, const relax_qmat &w, const void *out)
{
    return w.k % (2 * BK) == 0 && w.m % 4 == 0 && (w.group == 0 || w.group == 32) && (reinterpret_cast<uintptr_t>(x) & 15) == 0 &&
           (reinterpret_cast<uintptr_t>(w.q) & 3) == 0 && (reinterpret_cast<uintptr_t>(w.s) & 1) == 0 && (reinterpret_cast<uintptr_t>(out) & 7) == 0;
}

hipError_t launch_gemm_q3(const uint16_t *x, const relax_qmat &w, int n, uint16_t *out, hipStream_t stream)
{
    GemmArgs a = {};
    a.x = x, a.q = w.q, a.s = w.s, a.gshift = 0, a.n = n, a.m = w.m, a.k = w.k, a.epi = EPI_F16, a.out_f16 = out;
    const TilePlan p = tile_plan(w.m, w.k, n, EPI_F16);
    a.kb_per_split = w.k / BK;
    if (p.mf == 4) return launch_tile<2, 4, false, 4, 2, true>(a, stream, 1);
    if (p.nf == 4) return launch_tile<2, 4, false, 2, 2, true>(a, stream, 1);
    if (p.nf == 2) return launch_tile<2, 2, false, 2, 2, true>(a, stream, 1);
    return launch_tile<2, 1, false, 2, 2, true>(a, stream, 1);
}

hipError_t launch_gemm_mfma(const uint16_t *x, const relax_qmat &w, int n, int epi, uint16_t *out_f16, float *out_f32, const void *resid,
                            hipStream_t stream, float *partial, size_t partial_floats, const SkinnyFuse *fuse)
{
    GemmArgs a = {};
    a.wh = nullptr;
    a.x = x, a.q = w.q, a.s = w.s, a.gshift = gshift_of(w.group), a.n = n, a.m = w.m, a.k = w.k, a.epi = epi;
    a.out_f16 = out_f16, a.out_f32 = out_f32, a.resid = resid;
    TilePlan p = tile_plan(w.m, w.k, n, epi);
    if (p.splits > 1 && gemm_mfma_splits(w, n, epi, partial, partial_floats) == 1)
        p.splits = 1, p.kb_per_split = w.k / BK;                  // no workspace for the partial tiles: one pass over k
    if (fuse && p.splits < 2) return hipErrorInvalidValue;        // a folded light step needs the finishing pass
    a.partial = p.splits > 1 ? partial : nullptr;
    a.kb_per_split = p.kb_per_split;
    hipError_t e;
    const bool eight = g_waves_per_simd.load() == 2;
    if (p.m_big > 0 && p.splits == 1 && epi != EPI_SWIGLU) {
        // rows [0, m_big) on wide tiles, rows [m_big, m) on the narrow ones: two launches on the same stream
        GemmArgs b = a;
        b.m = p.m_big, b.ldm = w.m;
        e = eight ? launch_tile<2, 4, false, 4, 2>(b, stream, 1) : launch_tile<4, 4>(b, stream, 1);
        if (e != hipSuccess) return e;
        GemmArgs c = a;
        const size_t skip = (size_t)p.m_big;
        c.q = a.q + skip * (size_t)(w.k / 8), c.s = a.s + skip * (size_t)scales_per_row(w.k, a.gshift);
        c.m = w.m - p.m_big, c.ldm = w.m;
        if (c.out_f16) c.out_f16 = a.out_f16 + skip;
        if (c.out_f32) c.out_f32 = a.out_f32 + skip;
        if (c.resid) c.resid = (epi == EPI_RESID_F32) ? (const void *)((const uint16_t *)a.resid + skip) : (const void *)((const float *)a.resid + skip);
        return launch_tile<2, 4>(c, stream, 1);
    }
    if (p.mf == 4) e = eight ? launch_tile<2, 4, false, 4, 2>(a, stream, p.splits) : launch_tile<4, 4>(a, stream, p.splits);
    else if (p.nf == 4) e = launch_tile<2, 4>(a, stream, p.splits);        // 128 x 256: four wavefronts of 64 x 128 beat eight of 64 x 64 by 4 to 11 %
    else if (p.nf == 2) e = launch_tile<2, 2>(a, stream, p.splits);
    else e = launch_tile<2, 1>(a, stream, p.splits);
    if (e != hipSuccess || p.splits < 2) return e;
    return launch_skinny_finish(partial, p.splits, n, w.m, epi, out_f16, out_f32, resid, stream, fuse);
}

}  // namespace relax
