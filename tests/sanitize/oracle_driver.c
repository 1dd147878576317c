/* Runs every function of the CPU oracle on small ragged inputs.  Built by tests/test_sanitizers.py with
 * -fsanitize=address,undefined: the point is that no access leaves its buffer and no arithmetic is undefined; the
 * only numeric checks are that outputs are finite and that two invariants hold (probabilities sum to 1, a call on
 * rows of one prefill equals the same rows decoded one by one).  Buffers are malloc'ed at their exact size so that an
 * overrun lands in a red zone. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "relax_oracle.h"

static uint32_t lcg_state = 12345u;
static uint32_t lcg(void) { lcg_state = lcg_state * 1664525u + 1013904223u; return lcg_state; }
static float unit(void) { return (float)(lcg() >> 8) / 8388608.0f - 1.0f; }          /* [-1, 1) */

static uint16_t f16_bits(float v)       /* small positive normals and zero only: enough for scales and norm weights */
{
    if (v <= 0.0f) return 0;
    int e;
    float m = frexpf(v, &e);            /* v = m 2^e, m in [0.5, 1) */
    int be = e - 1 + 15;
    if (be <= 0) return 0;
    if (be >= 31) return 0x7BFF;
    return (uint16_t)((be << 10) | ((uint32_t)((m * 2.0f - 1.0f) * 1024.0f) & 0x3FF));
}

static void *xalloc(size_t bytes) { void *p = malloc(bytes ? bytes : 1); if (!p) { fprintf(stderr, "out of memory\n"); exit(2); } return p; }

static void check_finite(const float *v, size_t n, const char *what)
{
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(v[i])) { fprintf(stderr, "%s: element %zu is not finite\n", what, i); exit(1); }
}

typedef struct { uint32_t *q; uint16_t *s; int m, k, group; } qm;
static qm make_qmat(int m, int k, int group)
{
    qm w = {0};
    const int sg = (k + group - 1) / group;
    w.m = m, w.k = k, w.group = group;
    w.q = xalloc((size_t)m * (k / 8) * 4);
    w.s = xalloc((size_t)m * sg * 2);
    for (size_t i = 0; i < (size_t)m * (k / 8); ++i) w.q[i] = lcg() ^ (lcg() << 16);
    for (size_t i = 0; i < (size_t)m * sg; ++i) w.s[i] = f16_bits(0.002f + 0.01f * (unit() * 0.5f + 0.5f));
    return w;
}
static void free_qmat(qm *w) { free(w->q); free(w->s); }

int main(void)
{
    /* ---- decode exports and matmuls, k = 688 has a short last group for every group size ---- */
    const int groups[3] = {32, 64, 128};
    for (int gi = 0; gi < 3; ++gi) {
        const int m = 5, k = 688, n = 3, g = groups[gi];
        qm w = make_qmat(m, k, g);
        int8_t *codes = xalloc((size_t)m * k);
        float *dense = xalloc((size_t)m * k * 4), *x = xalloc((size_t)n * k * 4), *out = xalloc((size_t)n * m * 4);
        for (int i = 0; i < n * k; ++i) x[i] = unit();
        oracle_unpack_int4(w.q, m, k, codes);
        for (int i = 0; i < m * k; ++i) if (codes[i] < -8 || codes[i] > 7) { fprintf(stderr, "code out of range\n"); return 1; }
        oracle_dequantize_g(w.q, w.s, m, k, g, dense);
        oracle_dequant_matmul_g(x, w.q, w.s, m, k, g, out, n);
        check_finite(dense, (size_t)m * k, "dequantize_g");
        check_finite(out, (size_t)n * m, "dequant_matmul_g");
        if (g == 32) {
            oracle_dequantize(w.q, w.s, m, k, dense);
            oracle_dequant_matmul(x, w.q, w.s, m, k, out, n);
            check_finite(out, (size_t)n * m, "dequant_matmul");
        }
        free(codes), free(dense), free(x), free(out), free_qmat(&w);
    }
    {
        const int m = 7, k = 40, n = 2;
        uint16_t *wh = xalloc((size_t)m * k * 2);
        float *x = xalloc((size_t)n * k * 4), *out = xalloc((size_t)n * m * 4);
        for (int i = 0; i < m * k; ++i) wh[i] = f16_bits(0.5f + 0.4f * unit());
        for (int i = 0; i < n * k; ++i) x[i] = unit();
        oracle_half_matmul(x, wh, m, k, out, n);
        check_finite(out, (size_t)n * m, "half_matmul");
        free(wh), free(x), free(out);
    }

    /* ---- a tiny layer: hidden 64, 4 heads over 2 KV heads of 16, ffn 88 (k % 32 != 0 in the down projection) ---- */
    oracle_dims dm = {64, 4, 2, 16, 88, 1e-5f, 10000.0f, 12};
    const int H = dm.hidden, hd = dm.n_heads * dm.head_dim, gd = dm.n_kv_heads * dm.head_dim, F = dm.ffn, slots = 3;
    qm wqkv = make_qmat(hd + 2 * gd, H, 32), wo = make_qmat(H, hd, 32), wgu = make_qmat(2 * F, H, 32), wdown = make_qmat(H, F, 32);
    uint16_t *na = xalloc((size_t)H * 2), *nf = xalloc((size_t)H * 2);
    for (int i = 0; i < H; ++i) na[i] = f16_bits(1.0f + 0.1f * unit()), nf[i] = f16_bits(1.0f + 0.1f * unit());
    oracle_layer_weights lw = {{wqkv.q, wqkv.s, wqkv.m, wqkv.k, 32}, {wo.q, wo.s, wo.m, wo.k, 32}, {wgu.q, wgu.s, wgu.m, wgu.k, 32},
                               {wdown.q, wdown.s, wdown.m, wdown.k, 32}, na, nf};
    const size_t cache_elems = (size_t)slots * dm.kv_capacity * gd;
    float *kc = xalloc(cache_elems * 4), *vc = xalloc(cache_elems * 4), *kc2 = xalloc(cache_elems * 4), *vc2 = xalloc(cache_elems * 4);
    memset(kc, 0, cache_elems * 4), memset(vc, 0, cache_elems * 4), memset(kc2, 0, cache_elems * 4), memset(vc2, 0, cache_elems * 4);

    /* ragged call: 5 rows into slot 2, 1 row into slot 0, 3 rows into slot 1; then the first sequence again row by row */
    const int32_t q_lens[3] = {5, 1, 3}, kv_lens[3] = {5, 1, 3}, slot_of[3] = {2, 0, 1};
    const int n = 9;
    float *x = xalloc((size_t)n * H * 4), *out = xalloc((size_t)n * H * 4), *out1 = xalloc((size_t)H * 4);
    for (int i = 0; i < n * H; ++i) x[i] = unit();
    float *taps_mem[5];
    const size_t tap_elems[5] = {(size_t)n * H, (size_t)n * (hd + 2 * gd), (size_t)n * hd, (size_t)n * H, (size_t)n * F};
    for (int t = 0; t < 5; ++t) taps_mem[t] = xalloc(tap_elems[t] * 4);
    oracle_layer_taps taps = {taps_mem[0], taps_mem[1], taps_mem[2], taps_mem[3], taps_mem[4]};
    oracle_seqs sq = {3, q_lens, kv_lens, slot_of};
    if (oracle_decoder_layer_f32(&dm, &lw, x, kc, vc, &sq, out, n, &taps) != 0) { fprintf(stderr, "layer call rejected\n"); return 1; }
    check_finite(out, (size_t)n * H, "decoder_layer_f32");
    for (int t = 0; t < 5; ++t) check_finite(taps_mem[t], tap_elems[t], "layer taps");
    for (int r = 0; r < 5; ++r) {                       /* rows of the first sequence one by one: same values */
        const int32_t ql = 1, kl = r + 1, sl = 2;
        oracle_seqs one = {1, &ql, &kl, &sl};
        if (oracle_decoder_layer_f32(&dm, &lw, x + (size_t)r * H, kc2, vc2, &one, out1, 1, NULL) != 0) return 1;
        if (memcmp(out1, out + (size_t)r * H, (size_t)H * 4) != 0) { fprintf(stderr, "prefill row %d differs from its decode step\n", r); return 1; }
    }
    {   /* the fp16-input entry on the same call shape, and a call that must be rejected (capacity exceeded) */
        uint16_t *xh = xalloc((size_t)n * H * 2);
        for (int i = 0; i < n * H; ++i) xh[i] = f16_bits(0.5f + 0.49f * unit());
        memset(kc, 0, cache_elems * 4), memset(vc, 0, cache_elems * 4);
        if (oracle_decoder_layer(&dm, &lw, xh, kc, vc, &sq, out, n, NULL) != 0) return 1;
        check_finite(out, (size_t)n * H, "decoder_layer");
        const int32_t ql = 1, kl = dm.kv_capacity + 1, sl = 0;
        oracle_seqs bad = {1, &ql, &kl, &sl};
        if (oracle_decoder_layer(&dm, &lw, xh, kc, vc, &bad, out, 1, NULL) == 0) { fprintf(stderr, "a call beyond the cache capacity was accepted\n"); return 1; }
        free(xh);
    }

    /* ---- the pieces on their own ---- */
    {
        float *y = xalloc((size_t)n * H * 4);
        oracle_rmsnorm(x, na, y, n, H, dm.rms_eps);
        check_finite(y, (size_t)n * H, "rmsnorm");
        float v[16];
        for (int i = 0; i < 16; ++i) v[i] = unit();
        oracle_rope(v, 16, 11, dm.rope_base);
        check_finite(v, 16, "rope");
        float *qkv = xalloc((size_t)n * (hd + 2 * gd) * 4), *att = xalloc((size_t)n * hd * 4);
        for (int i = 0; i < n * (hd + 2 * gd); ++i) qkv[i] = unit();
        memset(kc, 0, cache_elems * 4), memset(vc, 0, cache_elems * 4);
        oracle_rope_append(qkv, &dm, kc, vc, &sq, n);
        /* probabilities [n, h, L_max]: rows of a query sum to 1 over its visible positions */
        float *probs = xalloc((size_t)n * dm.n_heads * dm.kv_capacity * 4);
        memset(probs, 0, (size_t)n * dm.n_heads * dm.kv_capacity * 4);
        oracle_attention(qkv, kc, vc, &dm, &sq, att, n, probs);
        check_finite(att, (size_t)n * hd, "attention");
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < dm.n_heads; ++j) {
                double sum = 0.0;
                for (int t = 0; t < dm.kv_capacity; ++t) sum += probs[((size_t)i * dm.n_heads + j) * dm.kv_capacity + t];
                if (fabs(sum - 1.0) > 1e-5) { fprintf(stderr, "probabilities of row %d head %d sum to %g\n", i, j, sum); return 1; }
            }
        float *gu = xalloc((size_t)n * 2 * F * 4), *a = xalloc((size_t)n * F * 4);
        for (int i = 0; i < n * 2 * F; ++i) gu[i] = 4.0f * unit();
        oracle_swiglu(gu, a, n, F);
        check_finite(a, (size_t)n * F, "swiglu");
        int32_t ids[9];
        oracle_argmax(out, n, H, ids);
        for (int i = 0; i < n; ++i) if (ids[i] < 0 || ids[i] >= H) return 1;
        free(y), free(qkv), free(att), free(probs), free(gu), free(a);
    }
    if (oracle_half_to_float(0x3C00) != 1.0f || oracle_num_threads() < 1) return 1;

    for (int t = 0; t < 5; ++t) free(taps_mem[t]);
    free(x), free(out), free(out1), free(kc), free(vc), free(kc2), free(vc2), free(na), free(nf);
    free_qmat(&wqkv), free_qmat(&wo), free_qmat(&wgu), free_qmat(&wdown);
    printf("oracle driver ok\n");
    return 0;
}
