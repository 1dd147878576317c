// Causal attention for calls with many rows per sequence (prefill): the contraction is dense, so it runs on
// MFMA, tiled over the KV length with the running (max, sum) rescaling of an online softmax.  In the paper's
// terms this is the attention operator lowered to a hand-written library kernel whose q length n and KV length
// L are runtime values (Relax, Sec. 4.2 custom attention pattern, Sec. 4.5 cross-level library dispatch,
// Sec. 5.1 dynamic sequence length); scores, softmax and accumulation are fp32.
//
// Mapping for gfx950 (v_mfma_f32_32x32x16_f16, 64-wide wavefronts):
//   - Everything is computed transposed, S^T = K Q^T and O^T = V^T P^T, so that a query is a COLUMN of the MFMA
//     result: lane l of a wavefront then owns query (l % 32) in every accumulator register.  The row maximum and
//     row sum of the softmax become in-lane reductions plus one exchange with lane l ^ 32, the rescaling of O is a
//     per-lane scalar, and the probabilities a lane holds after S^T are exactly the eight k-values the B operand
//     of the second product wants from it -- P never goes through LDS or a shuffle.
//   - K tile in LDS as [t][d]: the A operand of K Q^T is a 16-byte row read.  V tile in LDS as [t][d] too; the A
//     operand of V^T P^T needs eight t-values of one d per lane, which the LDS transpose read of gfx950
//     (ds_read_b64_tr_b16) delivers from the untransposed tile: inside a block of 16 lanes, lane r supplies the
//     address of 4 halfs and lane L receives half (L % 4) of the rows supplied by lanes L/4 + 4j, j = 0..3.
//     With lane r pointing at V[t0 + r/4][d0 + 4 (r%4)], lane L receives V[t0 + 0..3][d0 + L].
//   - A workgroup is 128 queries of one (sequence, head) on 8 wavefronts: 4 query groups of 32 x 2 groups along the
//     KV length (a wavefront takes every second 32-token sub-tile; the two states of a query group are merged
//     through LDS at the end).  The step count of the longest prefix sets the kernel time, and this halves it; fewer
//     queries per workgroup cost more than they give because every workgroup stages every K/V tile of its prefix.
//     A wavefront keeps its 32 queries' Q fragments in registers, O^T (32 x d fp32) in accumulators.  KV tiles of
//     64 tokens are staged through registers (the next tile's global loads are in flight during the MFMAs).
//   - Workgroups of the longest prefixes are first in dispatch order (causal work grows with the q position).
//   - Cache rows past a sequence's length are never read (loads are clamped to its last row); masked scores are
//     replaced, not multiplied, so stale cache contents cannot leak in.
#include "relax_common.h"

namespace relax {

namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kTB = 32;              // tokens per KV tile

struct SeqInfo {
    int32_t q_start, q_len, kv_len, slot;
};

__device__ inline SeqInfo seq_info(const SeqTable &st, int b)
{
    SeqInfo s;
    if (st.dev) {
        s.q_start = st.dev[b], s.q_len = st.dev[st.B + b], s.kv_len = st.dev[2 * st.B + b], s.slot = st.dev[3 * st.B + b];
    } else {
        s.q_start = s.q_len = s.kv_len = s.slot = 0;
#pragma unroll
        for (int j = 0; j < kInlineSeqs; ++j)
            if (j == b) s.q_start = st.q_start[j], s.q_len = st.q_len[j], s.kv_len = st.kv_len[j], s.slot = st.slot[j];
    }
    return s;
}

// LDS-only workgroup barrier: outstanding global loads (the next KV tile) stay in flight across it
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// grid: x = query head, y = q tile (reversed: longest prefix first), z = sequence
template <int D, int NWV, int NSUB, int TBS, int KVS>
__global__ __launch_bounds__(64 * NWV) void attn_prefill_kernel(const uint16_t *__restrict__ q, int q_stride,
                                                                 const uint16_t *__restrict__ kc, const uint16_t *__restrict__ vc,
                                                                 uint16_t *__restrict__ out, SeqTable st, int h, int g, int cap)
{
    // NWV wavefronts = QW query groups x KVS groups along the KV length: wavefront (qw, kg) owns queries qw WQ .. + WQ of the
    // workgroup and every KVS-th 32-token sub-tile (the longest prefix is then KVS times fewer steps per wavefront);
    // the KVS states of a query group are merged through LDS at the end.
    static_assert(TBS % KVS == 0 && NWV % KVS == 0, "sub-tiles are dealt round-robin to the KV groups");
    constexpr int QW = NWV / KVS;
    constexpr int kQB = QW * NSUB * 32;             // queries per workgroup
    constexpr int kPThreads = 64 * NWV, WQ = NSUB * 32;
    constexpr int KS = D / 16;       // k steps of K Q^T
    constexpr int DB = D / 32;       // 32-wide blocks of the head dimension in O^T
    constexpr int KP = D + 8;        // K tile pitch in halfs: 16-byte row reads of 32 rows hit distinct banks
    constexpr int VP = D + 32;       // V tile pitch in halfs: the 8-byte transpose reads of a 32-lane half hit distinct banks
    constexpr int TT = kTB * TBS;    // tokens staged per barrier pair: TBS sub-tiles of 32
    constexpr int PK = TT * (D / 8) / kPThreads;    // 16-byte packets per thread and tile, for K and for V
    constexpr int kTileHalfs = TT * KP + TT * VP;
    constexpr int kMergeFloats = KVS > 1 ? (KVS / 2) * QW * 64 * (NSUB * (DB * 16 + 2)) : 0;   // one merge round: half of the KV groups write
    constexpr int kSmemBytes = kTileHalfs * 2 > kMergeFloats * 4 ? kTileHalfs * 2 : kMergeFloats * 4;
    __shared__ __align__(16) unsigned char smem[kSmemBytes];
    uint16_t *const Ks = reinterpret_cast<uint16_t *>(smem), *const Vs = Ks + TT * KP;

    const SeqInfo si = seq_info(st, blockIdx.z);
    const int qt = gridDim.y - 1 - blockIdx.y;
    const int rows = min(kQB, si.q_len - qt * kQB);
    if (rows <= 0) return;                                        // uniform for the workgroup
    const int head = blockIdx.x, kvh = head / (h / g);
    const int past = si.kv_len - si.q_len;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, qw = wave % QW, kg = wave / QW;
    const int i32 = lane & 31, hf = lane >> 5;
    const int pos_block_max = past + qt * kQB + rows - 1;         // last token any query of the workgroup attends to
    const int wave_rows = min(WQ, rows - qw * WQ);              // <= 0: the wavefront only helps staging
    const int pos_wave_max = wave_rows > 0 ? past + qt * kQB + qw * WQ + wave_rows - 1 : -1;
    const float scale = 1.0f / sqrtf((float)D);

    // ---- Q fragments (B operand of K Q^T): lane owns query i32 of each 32-query sub-tile, 8 d-values per k step ----
    half8_t qf[NSUB][KS];
    int pos_q[NSUB];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const int local = qw * WQ + sub * 32 + i32;
        pos_q[sub] = past + qt * kQB + local;
        const int row = si.q_start + qt * kQB + min(local, rows - 1);
        const uint16_t *src = q + (size_t)row * q_stride + (size_t)head * D + hf * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[sub][ks] = *(const half8_t *)(src + ks * 16);
    }

    float16_t O[NSUB][DB];
    float m_run[NSUB], l_run[NSUB];
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        m_run[sub] = -INFINITY, l_run[sub] = 0.0f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) O[sub][db][v] = 0.0f;
    }

    // ---- KV tile staging ----
    const size_t slot_base = (size_t)si.slot * cap;
    const int t_last = si.kv_len - 1;
    u32x4_t kreg[PK], vreg[PK];
    auto tile_load = [&](int t0) {
#pragma unroll
        for (int p = 0; p < PK; ++p) {
            const int pk = tid + p * kPThreads, r = pk / (D / 8), c = pk % (D / 8);
            const size_t at = ((slot_base + min(t0 + r, t_last)) * g + kvh) * D + c * 8;
            kreg[p] = *(const u32x4_t *)(kc + at);
            vreg[p] = *(const u32x4_t *)(vc + at);
        }
    };
    auto tile_store = [&]() {
#pragma unroll
        for (int p = 0; p < PK; ++p) {
            const int pk = tid + p * kPThreads, r = pk / (D / 8), c = pk % (D / 8);
            *(u32x4_t *)(Ks + r * KP + c * 8) = kreg[p];
            *(u32x4_t *)(Vs + r * VP + c * 8) = vreg[p];
        }
    };

    // lane roles of the transpose read: lane r of a 16-lane block addresses V[.. + r/4][.. + 4 (r%4)]
    const int tr_row = hf * 4 + ((lane & 15) >> 2), tr_col = ((lane >> 4) & 1) * 16 + (lane & 3) * 4;

    tile_load(0);
    for (int tb = 0; tb <= pos_block_max; tb += TT) {
        tile_store();
        lds_barrier();
        tile_load(tb + TT);                                       // rows are clamped to the sequence: the tail re-reads its last row
#pragma unroll
        for (int u = 0; u < TBS; ++u) {
        const int t0 = tb + u * kTB;
        const uint16_t *Ku = Ks + u * kTB * KP, *Vu = Vs + u * kTB * VP;
        if (u % KVS == kg && t0 <= pos_wave_max) {
            // ---- S^T = K Q^T: 32 tokens x two 32-query sub-tiles ----
            float16_t S[NSUB];
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub)
#pragma unroll
                for (int v = 0; v < 16; ++v) S[sub][v] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const half8_t kf = *(const half8_t *)(Ku + i32 * KP + ks * 16 + hf * 8);
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) S[sub] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[sub][ks], S[sub], 0, 0, 0);
            }
            // ---- mask, online softmax; P^T packed as the B operand of the second product ----
            half8_t pf[NSUB][2];
#pragma unroll
            for (int sub = 0; sub < NSUB; ++sub) {
                float mx = -INFINITY;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = t0 + 8 * (v >> 2) + 4 * hf + (v & 3);
                    const float s = t <= pos_q[sub] ? S[sub][v] * scale : -INFINITY;
                    S[sub][v] = s;
                    mx = fmaxf(mx, s);
                }
                mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
                // The reference point of the exponentials only has to stay within reach of the true maximum: it is
                // moved (and O, l rescaled) when the maximum has grown by more than kSlack, so that most tiles skip the
                // rescaling of the 64 x d accumulator.  exp(kSlack) stays far inside fp16 for P and fp32 for l.
                constexpr float kSlack = 6.0f;
                const bool move = mx > m_run[sub] + kSlack;          // first tile: m_run = -inf -> always
                const float m_new = move ? mx : m_run[sub];          // finite from the first tile on: token 0 is visible
                // a KV group's first sub-tiles can be masked entirely for the earlier queries of the wavefront: no reference yet,
                // every weight is exp(-inf - 0) = 0 and the state stays empty
                const float m_ref = m_new == -INFINITY ? 0.0f : m_new;
                const float alpha = move ? __expf(m_run[sub] - m_ref) : 1.0f;      // exp(-inf) = 0 on the first tile
                float psum = 0.0f;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __expf(S[sub][v] - m_ref);
                    psum += p;
                    pf[sub][v >> 3][v & 7] = (_Float16)p;
                }
                l_run[sub] = l_run[sub] * alpha + psum;
                m_run[sub] = m_new;
                if (__any(move)) {
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) O[sub][db][v] *= alpha;
                }
            }
            // ---- O^T += V^T P^T ----
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const uint16_t *vp = Vu + (s2 * 16 + tr_row) * VP + db * 32 + tr_col;
                    const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t *)vp);
                    const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4_t *)(vp + 8 * VP));
                    const half8_t vf = __builtin_bit_cast(half8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                    for (int sub = 0; sub < NSUB; ++sub)
                        O[sub][db] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf[sub][s2], O[sub][db], 0, 0, 0);
                }
        }
        }
        lds_barrier();                                            // the tile is consumed: the next store may overwrite it
    }

    // ---- merge the KV groups of each query group: log2(KVS) rounds, the upper half of the groups hands its state to the lower half ----
    if (KVS > 1) {
        float *const mg = reinterpret_cast<float *>(smem);        // [writer wavefront][value][lane]: the tiles are consumed
        constexpr int kVals = NSUB * (DB * 16 + 2);
#pragma unroll
        for (int half = KVS / 2; half >= 1; half >>= 1) {
            if (kg >= half && kg < 2 * half) {
                float *dst = mg + ((size_t)((kg - half) * QW + qw) * kVals) * 64 + lane;
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) {
                    float *d2 = dst + (size_t)sub * (DB * 16 + 2) * 64;
                    d2[0] = m_run[sub], d2[64] = l_run[sub];
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) d2[(2 + db * 16 + v) * 64] = O[sub][db][v];
                }
            }
            __syncthreads();
            if (kg < half) {
                const float *src = mg + ((size_t)(kg * QW + qw) * kVals) * 64 + lane;
#pragma unroll
                for (int sub = 0; sub < NSUB; ++sub) {
                    const float *s2 = src + (size_t)sub * (DB * 16 + 2) * 64;
                    const float mb = s2[0], lb = s2[64];
                    const float mn = fmaxf(m_run[sub], mb);
                    const float ca = m_run[sub] == -INFINITY ? 0.0f : __expf(m_run[sub] - mn);
                    const float cb = mb == -INFINITY ? 0.0f : __expf(mb - mn);
                    l_run[sub] = l_run[sub] * ca + lb * cb;
                    m_run[sub] = mn;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int v = 0; v < 16; ++v) O[sub][db][v] = O[sub][db][v] * ca + s2[(2 + db * 16 + v) * 64] * cb;
                }
            }
            __syncthreads();
        }
        if (kg != 0) return;
    }

    // ---- normalise and store: lane holds query i32; register v of block db is d = 32 db + 8 (v/4) + 4 hf + v%4 ----
#pragma unroll
    for (int sub = 0; sub < NSUB; ++sub) {
        const int local = qw * WQ + sub * 32 + i32;
        const float l_tot = l_run[sub] + __shfl_xor(l_run[sub], 32, kWave);
        if (local >= rows) continue;
        const float inv = 1.0f / l_tot;
        uint16_t *dst = out + (size_t)(si.q_start + qt * kQB + local) * ((size_t)h * D) + (size_t)head * D;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int b4 = 0; b4 < 4; ++b4) {
                const int dd = db * 32 + b4 * 8 + hf * 4;
                const uint32_t w0 = f2h(O[sub][db][b4 * 4] * inv) | ((uint32_t)f2h(O[sub][db][b4 * 4 + 1] * inv) << 16);
                const uint32_t w1 = f2h(O[sub][db][b4 * 4 + 2] * inv) | ((uint32_t)f2h(O[sub][db][b4 * 4 + 3] * inv) << 16);
                *(uint2 *)(dst + dd) = make_uint2(w0, w1);
            }
    }
}

}  // namespace

bool attn_prefill_supported(const relax_layer_dims &dm) { return dm.head_dim == 128 || dm.head_dim == 64; }

hipError_t launch_attention_prefill(const uint16_t *q, int32_t q_stride, const relax_kv_cache &cache, const relax_layer_dims &dm,
                                    const SeqTable &st, uint16_t *out, hipStream_t stream)
{
    // 8 wavefronts = 4 query groups of 32 x 2 KV groups, tiles of 64 tokens.  Measured at n = 2048, 32 heads of 128: 69 us; without the
    // KV groups (8 x 32 or 4 x 32 queries) 82-84 us, 2 x 64 queries per workgroup (the first form of this kernel) 128 us, 64 queries per
    // workgroup in any split 93-117 us (every workgroup stages every K/V tile of its prefix).
    constexpr int kWaves = 8, kSub = 1, kKvGroups = 2;
    const int tiles = (st.q_max + kWaves / kKvGroups * kSub * 32 - 1) / (kWaves / kKvGroups * kSub * 32);
    const dim3 grid(dm.n_heads, tiles, st.B);
    if (dm.head_dim == 128)
        hipLaunchKernelGGL((attn_prefill_kernel<128, kWaves, kSub, kKvGroups, kKvGroups>), grid, dim3(64 * kWaves), 0, stream, q, q_stride, cache.k, cache.v,
                           out, st, dm.n_heads, dm.n_kv_heads, dm.kv_capacity);
    else if (dm.head_dim == 64)
        hipLaunchKernelGGL((attn_prefill_kernel<64, kWaves, kSub, kKvGroups, kKvGroups>), grid, dim3(64 * kWaves), 0, stream, q, q_stride, cache.k, cache.v,
                           out, st, dm.n_heads, dm.n_kv_heads, dm.kv_capacity);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace relax
