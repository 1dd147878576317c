// Persistent fused decode layer (n = 1): the whole layer of relax_decoder_layer in ONE launch.
//
// Why: at batch 1 the layer is a 114 MB weight stream plus 16 KB * L of KV cache and almost no
// arithmetic (Relax, Sec. 5.1: batch-1 decoding is the matrix-vector special case).  Measured on
// MI355X a streaming read sustains ~6.5 TB/s, a kernel boundary costs 1-2 us of ramp-up and tail,
// a memory round trip ~1-2 us and a grid barrier 2-4 us (9 us with release/acquire fences, which
// write back and invalidate the per-XCD L2s).  A layer is five dependent steps, so a step-per-kernel
// or barrier-per-step design spends most of its time waiting, not streaming.
//
// This kernel runs one workgroup per CU (all co-resident) and has NO grid barrier.  The steps are
// chained by the data itself: every value that crosses workgroups (q, the new k/v row, attention
// partials, attention output, x1, act) is published as one 8-byte word {payload, epoch tag} with a
// single write-through store (payload = one fp32 or two fp16), and consumers poll those words until
// the tag equals the epoch of this call -- one store latency plus one load latency per transition.
//
// Memory operations of a wavefront complete in order, so a poll issued behind a bulk weight request
// would wait for megabytes to land.  The wavefronts therefore have roles: six WORKERS stream weights
// (two trips of 8 KB in flight each, requested one step ahead -- weights do not depend on
// activations -- so HBM keeps streaming while the dependency chain is resolved) and do the
// contraction; two POLLERS fetch each step's input vector into LDS and never issue bulk loads.
// Roles meet at workgroup barriers whose fences cover LDS only, so a worker never has to drain its
// in-flight weight loads to pass one.
// This is the operator fusion of Sec. 4.2 taken to its end; the exchange buffers and the epoch
// counter are kernel scratch lifted into the caller's workspace (Sec. 4.4).
//
// Steps of a workgroup (each worker wavefront owns tiles wave_global, wave_global + W, ... of a step):
//   A  RMSNorm(x) -> QKV matvec -> rotary embedding -> q and the new k/v row published, k/v appended to the cache
//   B  attention items (KV head group, split of L), all eight wavefronts: online softmax over the cache; the
//      workgroup that owns split 0 of a head group merges that group's partials and publishes the head output
//   C  output projection + residual -> x1 published (and kept in registers for step E)
//   D  RMSNorm(x1) -> gate/up matvec -> SwiGLU -> act published
//   E  down projection + residual -> out (fp16)
#include <algorithm>

#include "q4_device.h"

namespace relax {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr int kWorkers = 6;                                 // wavefronts 0..5 stream weights, 6..7 poll inputs
constexpr int kPollLanes = (kWaves - kWorkers) * kWave;
constexpr int kPollN = 16;                                  // words a poller lane requests per round
constexpr int kSpinLimit = 1 << 18;                         // bounded polling: a wait that cannot complete sets the error flag
constexpr int kMaxTilesPerWave = 16;

// sync area (uint32 index): epoch counter, exit counter, sticky error flag -- each on its own 128-byte line
constexpr int kSyncEpoch = 0, kSyncExit = 32, kSyncError = 64, kSyncWords = 96;

typedef unsigned long long u64;

__device__ __forceinline__ void st_coh(uint32_t *p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t ld_coh(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t pack2h(float lo, float hi) { return (uint32_t)f2h(lo) | ((uint32_t)f2h(hi) << 16); }

// one published word: low half = payload bits (one fp32 or two fp16), high half = epoch of the call that wrote it
__device__ __forceinline__ void ll_store_bits(u64 *p, uint32_t bits, uint32_t epoch)
{
    __hip_atomic_store(p, (u64)bits | ((u64)epoch << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void ll_store(u64 *p, float v, uint32_t epoch) { ll_store_bits(p, __float_as_uint(v), epoch); }
__device__ __forceinline__ u64 ll_load(const u64 *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Poll N words (idx[i] < 0: skip) until all carry `epoch`; bits[i] receives the payload.  All loads of a
// round are in flight together.
template <int N>
__device__ __forceinline__ void ll_poll(const u64 *base, const int *idx, uint32_t epoch, uint32_t *bits, uint32_t *sync)
{
    int spins = 0;
    bool ok;
    do {
        u64 w[N];
#pragma unroll
        for (int i = 0; i < N; ++i) w[i] = idx[i] >= 0 ? ll_load(base + idx[i]) : ((u64)epoch << 32);
        ok = true;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            bits[i] = (uint32_t)w[i];
            ok = ok && ((uint32_t)(w[i] >> 32) == epoch);
        }
        if (!ok) {
            if (++spins > kSpinLimit) {
                st_coh(sync + kSyncError, 1u);
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
    } while (!ok);
}

// tile -> matrix rows.  Rotary step: two adjacent rotation pairs (t, t+d/2, t+1, t+1+d/2) or four v rows;
// SwiGLU step: (f, f+F, f+1, f+1+F); residual steps: two adjacent rows.
__device__ __forceinline__ void tile_rows(const DecodeLayerArgs &a, int epi, int tile, int *rows)
{
    if (epi == EPI_ROPE_KV) {
        const int d4 = a.d >> 2, nqk = (a.h + a.g) * d4;
        if (tile < nqk) {
            const int j = tile / d4, t = (tile - j * d4) * 2;
            rows[0] = j * a.d + t, rows[1] = rows[0] + (a.d >> 1), rows[2] = rows[0] + 1, rows[3] = rows[1] + 1;
        } else {
            rows[0] = (a.h + a.g) * a.d + 4 * (tile - nqk);
            rows[1] = rows[0] + 1, rows[2] = rows[0] + 2, rows[3] = rows[0] + 3;
        }
    } else if (epi == EPI_SWIGLU) {
        rows[0] = 2 * tile, rows[1] = rows[0] + a.F, rows[2] = rows[0] + 1, rows[3] = rows[1] + 1;
    } else {
        rows[0] = 2 * tile, rows[1] = rows[0] + 1, rows[2] = rows[0], rows[3] = rows[1];
    }
}

__device__ __forceinline__ int tiles_of_wave(int ntiles, int wave_global, int W)
{
    return wave_global < ntiles ? (ntiles - wave_global + W - 1) / W : 0;
}

// One step of the layer as the kernel's step loop sees it.
struct Step {
    DLMat M;
    int epi, mode, ntiles, nsub;      // nsub: trips per tile
};

__device__ __forceinline__ Step make_step(const DecodeLayerArgs &a, int st)
{
    Step s;
    s.M = st == 0 ? a.wqkv : st == 1 ? a.wo : st == 2 ? a.wgu : a.wdown;
    s.epi = st == 0 ? EPI_ROPE_KV : st == 1 ? EPI_RESID_F32 : st == 2 ? EPI_SWIGLU : EPI_RESID_F16;
    s.mode = (st == 1 || st == 3) ? 1 : 0;
    const int nchunks = (s.M.k + 2047) >> 11;
    s.ntiles = st == 0 ? (a.wqkv.m >> 2) : st == 2 ? (a.F >> 1) : (s.M.m >> 1);
    s.nsub = s.mode ? (nchunks + 3) >> 2 : (nchunks + 1) >> 1;
    return s;
}

// Trip su of a worker wavefront: rows and first chunk; trips past the wavefront's share point at tile 0 / chunk 0
// (every idle wavefront re-reads that same cache-resident address) and are not live.
__device__ __forceinline__ void trip_target(const DecodeLayerArgs &a, const Step &sp, int su, int nsu, int wave_global, int W,
                                            int *rows, int &chunk0)
{
    const bool live = su < nsu;
    const int j = su / sp.nsub, sub = su - j * sp.nsub;
    tile_rows(a, sp.epi, live ? wave_global + j * W : 0, rows);
    chunk0 = live ? sub * (sp.mode ? 4 : 2) : 0;
}

// Request the first two trips of a step (they are consumed after the step's input has arrived).
__device__ __forceinline__ void step_prefetch(const DecodeLayerArgs &a, const Step &sp, Slot &s0, Slot &s1, int wave_global, int W,
                                              int lane)
{
    const int nsu = tiles_of_wave(sp.ntiles, wave_global, W) * sp.nsub;
    int rows[4], chunk0;
    trip_target(a, sp, 0, nsu, wave_global, W, rows, chunk0);
    slot_load(s0, sp.M, rows, chunk0, sp.mode, lane);
    trip_target(a, sp, 1, nsu, wave_global, W, rows, chunk0);
    slot_load(s1, sp.M, rows, chunk0, sp.mode, lane);
}

// The trips of one step for one worker wavefront: s0 / s1 hold trips 0 and 1 on entry and are refilled two trips
// ahead.  The reduced sums of the wavefront's j-th tile go to res[4j..4j+3] in LDS; the caller's epilogue picks
// them up afterwards, so inside the loop the weight loads are the only vector-memory traffic in flight.
__device__ __forceinline__ void step_trips(const DecodeLayerArgs &a, const Step &sp, Slot &s0, Slot &s1, const uint16_t *xs,
                                           const float *corr, float *res, int wave_global, int W, int lane)
{
    const int nsu = tiles_of_wave(sp.ntiles, wave_global, W) * sp.nsub;
    float acc8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc8[e] = 0.0f;

    auto trip = [&](Slot &s, int su) {
        const int j = su / sp.nsub, sub = su - j * sp.nsub;
        slot_consume(s, sp.M, xs, corr, sub * (sp.mode ? 4 : 2), sp.mode, lane, su < nsu, acc8);
        int rows[4], chunk0;
        trip_target(a, sp, su + 2, nsu, wave_global, W, rows, chunk0);
        slot_load(s, sp.M, rows, chunk0, sp.mode, lane);
        if (su < nsu && sub == sp.nsub - 1) {
            float v[4];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                v[r] = sp.mode ? ((r < 2) ? acc8[r] + acc8[r + 2] + acc8[r + 4] + acc8[r + 6] : 0.0f) : acc8[r] + acc8[r + 4];
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = wave_sum(v[r]);
            if (lane == 0) {
#pragma unroll
                for (int r = 0; r < 4; ++r) res[j * 4 + r] = v[r];
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc8[e] = 0.0f;
        }
    };
#pragma unroll 1
    for (int su = 0; su < nsu; su += 2) {
        trip(s0, su);
        trip(s1, su + 1);
    }
}

// Pollers: fetch `nwords` consecutive published words into raw[] as fp32 (fmt 0: one fp32 per word, 1: two fp16
// per word).  kPollN loads per lane are in flight per round; a round is repeated until every tag matches.
__device__ __forceinline__ void poll_vector(const u64 *src, int nwords, int fmt, uint32_t epoch, float *raw, int plane, uint32_t *sync)
{
    for (int base = plane; base < nwords; base += kPollN * kPollLanes) {
        u64 w[kPollN];
        int spins = 0;
        bool ok;
        do {
#pragma unroll
            for (int i = 0; i < kPollN; ++i) {
                const int c = base + i * kPollLanes;
                w[i] = c < nwords ? ll_load(src + c) : ((u64)epoch << 32);
            }
            ok = true;
#pragma unroll
            for (int i = 0; i < kPollN; ++i) ok = ok && ((uint32_t)(w[i] >> 32) == epoch);
            if (!ok) {
                if (++spins > kSpinLimit) {
                    st_coh(sync + kSyncError, 1u);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
        } while (!ok);
#pragma unroll
        for (int i = 0; i < kPollN; ++i) {
            const int c = base + i * kPollLanes;
            if (c < nwords) {
                const uint32_t bits = (uint32_t)w[i];
                if (fmt == 0) {
                    raw[c] = __uint_as_float(bits);
                } else {
                    raw[2 * c] = h2f((uint16_t)(bits & 0xFFFFu));
                    raw[2 * c + 1] = h2f((uint16_t)(bits >> 16));
                }
            }
        }
    }
}

// All eight wavefronts: raw[] (fp32, k values, already in LDS and fenced by a barrier) -> fp16 matvec layout in
// xs[] (+ per-group offset terms), optionally RMS-normalised with the fp16 weights wn[] (also in LDS).
__device__ __forceinline__ void stage_from_raw(const float *raw, const uint16_t *wn, bool norm, int k, float eps, uint16_t *xs,
                                               float *corr, float *red, int tid)
{
    const int kpad = ((k + 2047) >> 11) << 11, lane = tid & 63, wave = tid >> 6;
    float ss = 0.0f;
    if (norm)
        for (int c = tid; c < k; c += kThreads) ss += raw[c] * raw[c];
    ss = wave_sum(ss);
    if (lane == 0) red[wave] = ss;
    wg_barrier();
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) tot += red[w];
    const float inv = norm ? 1.0f / sqrtf(tot / (float)k + eps) : 1.0f;
    for (int c = tid; c < kpad; c += kThreads) {
        float v = 0.0f;
        if (c < k) v = norm ? raw[c] * inv * h2f(wn[c]) : raw[c];
        xs[fast_off(c)] = f2h(v);
    }
    wg_barrier();
    for (int gi = tid; gi < (k >> 5); gi += kThreads) corr[gi] = group_corr(xs, gi);
    wg_barrier();
}

__device__ __forceinline__ void unpack8(const uint4 &raw, float *f)
{
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[2 * j] = h2f((uint16_t)(w[j] & 0xFFFFu));
        f[2 * j + 1] = h2f((uint16_t)(w[j] >> 16));
    }
}

// Step B for one (head group, split) item, whole workgroup.  K/V of past tokens stream from the cache; the
// row of this call's token comes from the published k/v (it may not have reached the cache yet).
template <int D, int REP>
__device__ __forceinline__ void attention_item(const DecodeLayerArgs &a, int item, uint32_t epoch, float *sm, float *smq, float *smkv,
                                               int tid)
{
    constexpr int LPT = D / 8, TPW = kWave / LPT, U = 4;
    const int L = a.pos + 1, rep = a.h / a.g, subs = rep / REP;
    const int hg = item / a.splits, split = item - hg * a.splits;
    const int kvh = hg / subs, head0 = kvh * rep + (hg - kvh * subs) * REP;
    const int t_begin = split * a.chunk, t_end = min(L, t_begin + a.chunk);
    const int lane = tid & 63, wave = tid >> 6, sub = lane / LPT, e0 = (lane % LPT) * 8;
    const float inv_sqrt_d = 1.0f / sqrtf((float)D);
    const size_t slot_base = (size_t)a.slot * a.cap;
    const int stride = kWaves * TPW;
    const bool poller = wave >= kWorkers;

    uint4 kraw[U], vraw[U];
    const int t_first = t_begin + wave * TPW + sub;
    auto request = [&](int t0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * stride;
            if (t < t_end && t != a.pos) {
                const size_t at = ((slot_base + t) * a.g + kvh) * D + e0;
                kraw[u] = *(const uint4 *)(a.kcache + at);
                vraw[u] = *(const uint4 *)(a.vcache + at);
            }
        }
    };
    if (poller) {
        // q of the REP heads and the new k/v row of this KV head (two fp16 per word), shared through LDS
        const int plane = tid - kWorkers * kWave, nq = REP * D / 2, nw = nq + D;
        for (int c = plane; c < nw; c += kPollLanes) {
            int ix[1];
            uint32_t bits[1];
            const u64 *src;
            float *dst;
            if (c < nq) src = a.q_ll, ix[0] = head0 * D / 2 + c, dst = smq + 2 * c;
            else if (c < nq + D / 2) src = a.knew_ll, ix[0] = kvh * D / 2 + (c - nq), dst = smkv + 2 * (c - nq);
            else src = a.vnew_ll, ix[0] = kvh * D / 2 + (c - nq - D / 2), dst = smkv + D + 2 * (c - nq - D / 2);
            ll_poll<1>(src, ix, epoch, bits, a.sync);
            dst[0] = h2f((uint16_t)(bits[0] & 0xFFFFu));
            dst[1] = h2f((uint16_t)(bits[0] >> 16));
        }
    } else {
        request(t_first);          // workers: the first K/V tokens go out before q is known
    }
    wg_barrier();
    if (poller) request(t_first);

    float qf[REP][8], acc[REP][8], m[REP], l[REP];
#pragma unroll
    for (int r = 0; r < REP; ++r) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[r][e] = smq[r * D + e0 + e], acc[r][e] = 0.0f;
        m[r] = -INFINITY, l[r] = 0.0f;
    }
    for (int t0 = t_first; t0 < t_end; t0 += stride * U) {
        if (t0 != t_first) request(t0);    // the first round went out before the barrier; eight wavefronts overlap the rest
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * stride;
            if (t < t_end) {
                float kf[8], vf[8];
                if (t == a.pos) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) kf[e] = smkv[e0 + e], vf[e] = smkv[D + e0 + e];
                } else {
                    unpack8(kraw[u], kf);
                    unpack8(vraw[u], vf);
                }
#pragma unroll
                for (int r = 0; r < REP; ++r) {
                    float dot = 0.0f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) dot += qf[r][e] * kf[e];
#pragma unroll
                    for (int off = LPT / 2; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, kWave);
                    const float s = dot * inv_sqrt_d, mn = fmaxf(m[r], s);
                    const float ca = __expf(m[r] - mn), p = __expf(s - mn);
                    l[r] = l[r] * ca + p;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[r][e] = acc[r][e] * ca + p * vf[e];
                    m[r] = mn;
                }
            }
        }
    }
    // lanes that own the same 8 elements merge inside the wavefront, wavefronts merge through LDS
#pragma unroll
    for (int r = 0; r < REP; ++r) {
#pragma unroll
        for (int off = LPT; off < kWave; off <<= 1) {
            const float mb = __shfl_xor(m[r], off, kWave), lb = __shfl_xor(l[r], off, kWave);
            const float mn = fmaxf(m[r], mb);
            const float sa = (m[r] == -INFINITY) ? 0.0f : __expf(m[r] - mn), sb = (mb == -INFINITY) ? 0.0f : __expf(mb - mn);
            l[r] = l[r] * sa + lb * sb;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] = acc[r][e] * sa + __shfl_xor(acc[r][e], off, kWave) * sb;
            m[r] = mn;
        }
        if (lane < LPT) {
            float *dst = sm + (wave * REP + r) * (D + 2);
#pragma unroll
            for (int e = 0; e < 8; ++e) dst[e0 + e] = acc[r][e];
            if (lane == 0) dst[D] = m[r], dst[D + 1] = l[r];
        }
    }
    wg_barrier();
    // one thread per pair of output elements
    for (int idx = tid; idx < REP * D / 2; idx += kThreads) {
        const int r = idx / (D / 2), e = (idx - r * (D / 2)) * 2;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, sm[(w * REP + r) * (D + 2) + D]);
        float n0 = 0.0f, n1 = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float *src = sm + (w * REP + r) * (D + 2);
            const float sc = (src[D] == -INFINITY) ? 0.0f : __expf(src[D] - mm);
            n0 += src[e] * sc, n1 += src[e + 1] * sc, den += src[D + 1] * sc;
        }
        if (a.splits == 1) {
            ll_store_bits(a.attn_ll + ((size_t)(head0 + r) * D + e) / 2, pack2h(n0 / den, n1 / den), epoch);   // nothing to merge
        } else {
            u64 *dst = a.part_ll + ((size_t)(head0 + r) * a.splits + split) * (D + 2);    // [head][split][D+2] fp32 words
            ll_store(dst + e, n0, epoch), ll_store(dst + e + 1, n1, epoch);
            if (e == 0) ll_store(dst + D, mm, epoch), ll_store(dst + D + 1, den, epoch);
        }
    }
    wg_barrier();                                                  // sm, smq, smkv are reused by the next item
}

// Softmax merge of the splits of one head group: run by the pollers of the workgroup that owns its split 0, after
// all of that workgroup's own items.  One lane per pair of output elements.
template <int D, int REP>
__device__ __forceinline__ void attention_merge(const DecodeLayerArgs &a, int hg, uint32_t epoch, int plane)
{
    constexpr int SB = kPollN / 4;                                  // splits polled together: 4 words each
    const int rep = a.h / a.g, subs = rep / REP;
    const int kvh = hg / subs, head0 = kvh * rep + (hg - kvh * subs) * REP;
    for (int idx = plane; idx < REP * D / 2; idx += kPollLanes) {
        const int r = idx / (D / 2), e = (idx - r * (D / 2)) * 2;
        const u64 *src = a.part_ll + (size_t)(head0 + r) * a.splits * (D + 2);
        float mm = -INFINITY, n0 = 0.0f, n1 = 0.0f, den = 0.0f;
        for (int s0 = 0; s0 < a.splits; s0 += SB) {
            int ix[kPollN];
            uint32_t v[kPollN];
#pragma unroll
            for (int j = 0; j < SB; ++j) {
                const bool on = s0 + j < a.splits;
                const int at = (s0 + j) * (D + 2);
                ix[4 * j] = on ? at + e : -1, ix[4 * j + 1] = on ? at + e + 1 : -1;
                ix[4 * j + 2] = on ? at + D : -1, ix[4 * j + 3] = on ? at + D + 1 : -1;
            }
            ll_poll<kPollN>(src, ix, epoch, v, a.sync);
#pragma unroll
            for (int j = 0; j < SB; ++j) {
                if (s0 + j < a.splits) {
                    const float ms = __uint_as_float(v[4 * j + 2]), mn = fmaxf(mm, ms);
                    const float sa = (mm == -INFINITY) ? 0.0f : __expf(mm - mn), sb = __expf(ms - mn);
                    n0 = n0 * sa + __uint_as_float(v[4 * j]) * sb;
                    n1 = n1 * sa + __uint_as_float(v[4 * j + 1]) * sb;
                    den = den * sa + __uint_as_float(v[4 * j + 3]) * sb;
                    mm = mn;
                }
            }
        }
        ll_store_bits(a.attn_ll + ((size_t)(head0 + r) * D + e) / 2, pack2h(n0 / den, n1 / den), epoch);
    }
}

template <int D, int REP>
__global__ __launch_bounds__(kThreads) void decode_layer_kernel(DecodeLayerArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ float red[kWaves];
    uint16_t *xs = (uint16_t *)lds;
    float *corr = (float *)(lds + a.lds_corr);
    float *raw = (float *)(lds + a.lds_raw);
    uint16_t *wn_attn = (uint16_t *)(lds + a.lds_wn), *wn_ffn = wn_attn + a.H;
    float *sm = (float *)(lds + a.lds_attn);
    float *smq = sm + kWaves * REP * (D + 2);
    float *smkv = smq + REP * D;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool poller = wave >= kWorkers;
    const int plane = tid - kWorkers * kWave;                        // poller lane 0..127
    float *res = (float *)(lds + a.lds_res) + (poller ? 0 : wave) * (kMaxTilesPerWave * 4);
    const int nb = gridDim.x, W = nb * kWorkers, wave_global = poller ? 0x7fffffff : blockIdx.x * kWorkers + wave;
    uint32_t *sync = a.sync;
    auto stamp = [&](int i) {
        if (a.trace && tid == 0) a.trace[blockIdx.x * 16 + i] = wall_clock64();
    };
    stamp(0);
    const int hd2 = a.d >> 1, d4 = a.d >> 2, nqk = (a.h + a.g) * d4;

    Slot s0, s1;                                                    // the two weight trips a worker keeps in flight
    float4 cs = make_float4(1.0f, 0.0f, 1.0f, 0.0f);                // rotary (cos, sin) x2 of the lane's rotary-step tile
    uint32_t xres = 0;                                              // residual input of the lane's output-projection tile
    if (!poller) {
        const Step sp = make_step(a, 0);
        step_prefetch(a, sp, s0, s1, wave_global, W, lane);
        const int t = wave_global + lane * W;
        if (lane < tiles_of_wave(sp.ntiles, wave_global, W) && t < nqk)
            cs = *(const float4 *)(a.rope + ((size_t)a.pos * hd2 + (t % d4) * 2) * 2);
        if (lane < tiles_of_wave(a.wo.m >> 1, wave_global, W)) xres = *(const uint32_t *)(a.x + 2 * t);
    } else {
        // pollers bring in the layer input and both norm weight vectors (8 fp16 per load, four passes in flight)
        for (int base = plane; base < (a.H >> 3); base += 4 * kPollLanes) {
            uint4 xr[4], wa[4], wf[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c8 = min(base + i * kPollLanes, (a.H >> 3) - 1);
                xr[i] = *(const uint4 *)(a.x + c8 * 8);
                wa[i] = *(const uint4 *)(a.norm_attn + c8 * 8);
                wf[i] = *(const uint4 *)(a.norm_ffn + c8 * 8);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c8 = base + i * kPollLanes;
                if (c8 < (a.H >> 3)) {
                    float f[8];
                    unpack8(xr[i], f);
#pragma unroll
                    for (int e = 0; e < 8; ++e) raw[c8 * 8 + e] = f[e];
                    *(uint4 *)(wn_attn + c8 * 8) = wa[i];
                    *(uint4 *)(wn_ffn + c8 * 8) = wf[i];
                }
            }
        }
    }
    const uint32_t epoch = ld_coh(sync + kSyncEpoch) + 1u;
    const size_t tok = ((size_t)a.slot * a.cap + a.pos) * (size_t)(a.g * a.d);
    float x1keep[2] = {0.0f, 0.0f};

    // ---- the four weight steps (0: QKV, 1: output projection, 2: gate/up, 3: down) run through ONE loop body;
    //      attention sits between steps 0 and 1 ----------------------------------------------------------------
#pragma unroll 1
    for (int st = 0; st < 4; ++st) {
        const Step sp = make_step(a, st);
        if (st == 1) {
            const int groups = a.g * ((a.h / a.g) / REP), items = groups * a.splits;
            for (int item = blockIdx.x; item < items; item += nb) attention_item<D, REP>(a, item, epoch, sm, smq, smkv, tid);
            stamp(2);
            if (poller && a.splits > 1)
                for (int item = blockIdx.x; item < items; item += nb)
                    if (item % a.splits == 0) attention_merge<D, REP>(a, item / a.splits, epoch, plane);
            stamp(3);
            if (!poller) step_prefetch(a, sp, s0, s1, wave_global, W, lane);   // not held across attention: registers
        }
        // input of the step: pollers fetch it into raw[] (step 0: already there), everybody stages it
        if (poller && st > 0) {
            const u64 *src = st == 1 ? a.attn_ll : st == 2 ? a.x1_ll : a.act_ll;
            poll_vector(src, st == 2 ? sp.M.k : sp.M.k >> 1, st == 2 ? 0 : 1, epoch, raw, plane, sync);
        }
        wg_barrier();
        const bool norm = (st == 0 || st == 2);
        stage_from_raw(raw, st == 0 ? wn_attn : wn_ffn, norm, sp.M.k, a.eps, xs, corr, red, tid);
        stamp(4 + 2 * st);
        if (!poller) {
            step_trips(a, sp, s0, s1, xs, corr, res, wave_global, W, lane);
            if (st == 1 || st == 2) {
                const Step nx = make_step(a, st + 1);                // the next step's first trips go out now
                step_prefetch(a, nx, s0, s1, wave_global, W, lane);
            }
            if (lane < tiles_of_wave(sp.ntiles, wave_global, W)) {
                const int tile = wave_global + lane * W;
                const float v0 = res[lane * 4], v1 = res[lane * 4 + 1], v2 = res[lane * 4 + 2], v3 = res[lane * 4 + 3];
                if (st == 0) {
                    if (tile < nqk) {
                        const int j = tile / d4, t = (tile - j * d4) * 2;
                        const uint32_t lo = pack2h(v0 * cs.x - v1 * cs.y, v2 * cs.z - v3 * cs.w);     // elements t, t+1
                        const uint32_t hi = pack2h(v0 * cs.y + v1 * cs.x, v2 * cs.w + v3 * cs.z);     // t+d/2, t+d/2+1
                        if (j < a.h) {
                            u64 *qd = a.q_ll + ((size_t)j * a.d + t) / 2;
                            ll_store_bits(qd, lo, epoch), ll_store_bits(qd + (hd2 >> 1), hi, epoch);
                        } else {
                            const size_t at = (size_t)(j - a.h) * a.d + t;
                            ll_store_bits(a.knew_ll + at / 2, lo, epoch), ll_store_bits(a.knew_ll + at / 2 + (hd2 >> 1), hi, epoch);
                            uint32_t *kc = (uint32_t *)(a.kcache + tok + at);
                            st_coh(kc, lo), st_coh(kc + (hd2 >> 1), hi);
                        }
                    } else {
                        const size_t at = 4 * (size_t)(tile - nqk);
                        const uint32_t lo = pack2h(v0, v1), hi = pack2h(v2, v3);
                        ll_store_bits(a.vnew_ll + at / 2, lo, epoch), ll_store_bits(a.vnew_ll + at / 2 + 1, hi, epoch);
                        uint32_t *vc = (uint32_t *)(a.vcache + tok + at);
                        st_coh(vc, lo), st_coh(vc + 1, hi);
                    }
                } else if (st == 1) {
                    x1keep[0] = h2f((uint16_t)(xres & 0xFFFFu)) + v0;
                    x1keep[1] = h2f((uint16_t)(xres >> 16)) + v1;
                    ll_store(a.x1_ll + 2 * tile, x1keep[0], epoch);
                    ll_store(a.x1_ll + 2 * tile + 1, x1keep[1], epoch);
                } else if (st == 2) {
                    ll_store_bits(a.act_ll + tile, pack2h(v0 / (1.0f + expf(-v0)) * v1, v2 / (1.0f + expf(-v2)) * v3), epoch);
                } else {
                    *(uint32_t *)(a.out + 2 * tile) = pack2h(x1keep[0] + v0, x1keep[1] + v1);
                }
            }
        }
        stamp(5 + 2 * st);
    }

    // ---- the last workgroup out advances the epoch for the next call ---------------------------------------------
    wg_barrier();
    if (tid == 0) {
        const uint32_t old = __hip_atomic_fetch_add(sync + kSyncExit, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == (uint32_t)nb) {
            st_coh(sync + kSyncEpoch, epoch);
            st_coh(sync + kSyncExit, 0u);
        }
    }
}

__global__ void sync_clear_kernel(uint32_t *p, size_t count)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// LDS plan: staged vector | per-group terms | raw fp32 input | norm weights | attention merge area + q + new k/v | tile results
struct LdsPlan {
    int corr, raw, wn, attn, res, total;
};

LdsPlan lds_plan(int H, int hd, int F, int D, int REP)
{
    const int kmax = std::max(std::max(H, hd), F);
    const int kpad = ((kmax + 2047) / 2048) * 2048;
    LdsPlan p;
    p.corr = kpad * 2;
    p.raw = p.corr + ((kmax / 32 + 63) / 64) * 64 * 4;
    p.wn = p.raw + ((kmax + 63) / 64) * 64 * 4;
    p.attn = p.wn + 2 * H * 2;
    p.res = p.attn + (kWaves * REP * (D + 2) + REP * D + 2 * D) * 4;
    p.total = p.res + kWorkers * kMaxTilesPerWave * 4 * 4;
    return p;
}

constexpr int kLdsLimit = 160 * 1024 - 1024;

}  // namespace

size_t decode_layer_sync_bytes(const relax_layer_dims &) { return sizeof(uint32_t) * (size_t)kSyncWords; }
size_t decode_layer_error_offset() { return sizeof(uint32_t) * (size_t)kSyncError; }

// Zero the sync area and every exchange buffer (tag 0 is never a valid epoch).
hipError_t launch_sync_clear(void *base, size_t bytes, hipStream_t stream)
{
    hipLaunchKernelGGL(sync_clear_kernel, dim3(64), dim3(256), 0, stream, (uint32_t *)base, bytes / sizeof(uint32_t));
    return hipGetLastError();
}

// Whether the fused kernel can serve this call (else the caller falls back to the step-by-step kernels).
bool decode_layer_eligible(const relax_layer_dims &dm, const relax_layer_weights &w, int n, int B, int n_cus)
{
    if (n != 1 || B != 1 || n_cus < 8) return false;
    const relax_qmat *mats[4] = {&w.wqkv, &w.wo, &w.wgu, &w.wdown};
    for (const relax_qmat *m : mats)
        if (m->k % kGroup != 0 || (reinterpret_cast<uintptr_t>(m->q) & 15) != 0 || m->k > kMaxK) return false;
    if (dm.hidden % 8 != 0 || dm.ffn % 2 != 0) return false;
    if ((reinterpret_cast<uintptr_t>(w.norm_attn) & 15) != 0 || (reinterpret_cast<uintptr_t>(w.norm_ffn) & 15) != 0) return false;
    const int W = n_cus * kWorkers;
    const int tiles[4] = {w.wqkv.m / 4, w.wo.m / 2, dm.ffn / 2, w.wdown.m / 2};
    for (int t : tiles)
        if ((t + W - 1) / W > kMaxTilesPerWave) return false;
    if (w.wqkv.m % 4 != 0 || w.wo.m % 2 != 0 || w.wdown.m % 2 != 0 || w.wo.m != w.wdown.m) return false;
    if (lds_plan(dm.hidden, dm.n_heads * dm.head_dim, dm.ffn, dm.head_dim, 2).total > kLdsLimit) return false;
    return true;
}

template <int D, int REP>
static hipError_t launch_dl(DecodeLayerArgs &a, int n_cus, hipStream_t stream)
{
    const LdsPlan p = lds_plan(a.H, a.wo.k, a.F, D, REP);
    a.lds_corr = p.corr, a.lds_raw = p.raw, a.lds_wn = p.wn, a.lds_attn = p.attn, a.lds_res = p.res;
    // asking for more than half of the CU's 160 KB keeps the grid at exactly one workgroup per CU
    const int total = std::max(p.total, 84 * 1024);
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)decode_layer_kernel<D, REP>, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    a.nblocks = n_cus;
    hipLaunchKernelGGL((decode_layer_kernel<D, REP>), dim3(n_cus), dim3(kThreads), total, stream, a);
    return hipGetLastError();
}

hipError_t launch_decode_layer(DecodeLayerArgs &a, int n_cus, hipStream_t stream)
{
    const int rep = a.h / a.g;
    // query heads that share one K/V load
    const int REP = (rep % 2 == 0) ? 2 : 1;
    // attention plan: one item per workgroup when L is long enough; chunks are multiples of 64 tokens
    const int groups = a.g * (rep / REP), L = a.pos + 1;
    int splits = n_cus / groups;
    if (splits < 1) splits = 1;
    if (splits > kFusedMaxSplits) splits = kFusedMaxSplits;
    const int chunk = ((L + splits - 1) / splits + 63) / 64 * 64;
    a.chunk = chunk;
    a.splits = (L + chunk - 1) / chunk;
    if (a.d == 128) return REP == 2 ? launch_dl<128, 2>(a, n_cus, stream) : launch_dl<128, 1>(a, n_cus, stream);
    return REP == 2 ? launch_dl<64, 2>(a, n_cus, stream) : launch_dl<64, 1>(a, n_cus, stream);
}

}  // namespace relax
