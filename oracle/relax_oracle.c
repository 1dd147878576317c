/*
 * relax_oracle.c -- plain CPU reference for the int4 Llama-style decoder layer.
 * TEST INFRASTRUCTURE ONLY; see relax_oracle.h for scope, conventions and the
 * passages of the paper (Relax, arXiv 2311.02103) that fix the calling rules.
 *
 * Every function is the written-out definition: scalar loops, fp32, ascending
 * index order.  OpenMP pragmas only distribute independent outputs.
 */
#include "relax_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int32_t oracle_num_threads(void)
{
#ifdef _OPENMP
    return (int32_t)omp_get_max_threads();
#else
    return 1;
#endif
}

/* IEEE 754 binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits.        */
float oracle_half_to_float(uint16_t bits)
{
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 10) & 0x1F;
    int frac = bits & 0x3FF;
    float mag;
    if (expo == 0) {
        mag = ldexpf((float)frac, -24);                 /* zero / subnormal  */
    } else if (expo == 31) {
        mag = frac ? NAN : INFINITY;
    } else {
        mag = ldexpf((float)(1024 + frac), expo - 25);  /* (1+f/1024)*2^(e-15) */
    }
    return sign ? -mag : mag;
}

/* scales per row: one per `group` consecutive columns, the last group short when group does not divide k */
static int32_t groups_per_row(int32_t k, int32_t group) { return (k + group - 1) / group; }
static int32_t group_of(int32_t group) { return group > 0 ? group : 32; }     /* 0 in a descriptor reads as 32 */

/* code of element (r,c): word r*(k/8)+c/8, bits 4*(c%8)..4*(c%8)+3          */
static int nibble_code(const uint32_t *qweight, int32_t k, int32_t r, int32_t c)
{
    uint32_t word = qweight[(size_t)r * (size_t)(k / 8) + (size_t)(c / 8)];
    return (int)((word >> (4 * (c % 8))) & 0xFu);
}

void oracle_unpack_int4(const uint32_t *qweight, int32_t m, int32_t k, int8_t *out)
{
    for (int32_t r = 0; r < m; ++r)
        for (int32_t c = 0; c < k; ++c)
            out[(size_t)r * k + c] = (int8_t)(nibble_code(qweight, k, r, c) - 8);
}

static void dequant_row(const uint32_t *qweight, const uint16_t *scales,
                        int32_t k, int32_t group, int32_t r, float *row)
{
    int32_t G = groups_per_row(k, group);
    for (int32_t c = 0; c < k; ++c) {
        int q = nibble_code(qweight, k, r, c) - 8;
        float s = oracle_half_to_float(scales[(size_t)r * G + c / group]);
        row[c] = (float)q * s;
    }
}

void oracle_dequantize_g(const uint32_t *qweight, const uint16_t *scales,
                         int32_t m, int32_t k, int32_t group, float *out)
{
    group = group_of(group);
#pragma omp parallel for schedule(static)
    for (int32_t r = 0; r < m; ++r)
        dequant_row(qweight, scales, k, group, r, out + (size_t)r * k);
}

void oracle_dequantize(const uint32_t *qweight, const uint16_t *scales,
                       int32_t m, int32_t k, float *out)
{
    oracle_dequantize_g(qweight, scales, m, k, 32, out);
}

void oracle_dequant_matmul(const float *x, const uint32_t *qweight, const uint16_t *scales,
                           int32_t m, int32_t k, float *out, int32_t n)
{
    oracle_dequant_matmul_g(x, qweight, scales, m, k, 32, out, n);
}

void oracle_dequant_matmul_g(const float *x, const uint32_t *qweight, const uint16_t *scales,
                             int32_t m, int32_t k, int32_t group, float *out, int32_t n)
{
    group = group_of(group);
#pragma omp parallel
    {
        float *row = (float *)malloc(sizeof(float) * (size_t)(k > 0 ? k : 1));
#pragma omp for schedule(static)
        for (int32_t r = 0; r < m; ++r) {
            dequant_row(qweight, scales, k, group, r, row); /* W[r, :]        */
            for (int32_t i = 0; i < n; ++i) {
                const float *xi = x + (size_t)i * k;
                float acc = 0.0f;
                for (int32_t c = 0; c < k; ++c)
                    acc += xi[c] * row[c];
                out[(size_t)i * m + r] = acc;
            }
        }
        free(row);
    }
}

void oracle_half_matmul(const float *x, const uint16_t *w, int32_t m, int32_t k,
                        float *out, int32_t n)
{
#pragma omp parallel for schedule(static)
    for (int32_t r = 0; r < m; ++r) {
        for (int32_t i = 0; i < n; ++i) {
            const float *xi = x + (size_t)i * k;
            float acc = 0.0f;
            for (int32_t c = 0; c < k; ++c)
                acc += xi[c] * oracle_half_to_float(w[(size_t)r * k + c]);
            out[(size_t)i * m + r] = acc;
        }
    }
}

void oracle_rmsnorm(const float *x, const uint16_t *w, float *y,
                    int32_t n, int32_t H, float eps)
{
    for (int32_t i = 0; i < n; ++i) {
        const float *xi = x + (size_t)i * H;
        float ss = 0.0f;
        for (int32_t j = 0; j < H; ++j)
            ss += xi[j] * xi[j];
        float ms = ss / (float)H;
        float inv = 1.0f / sqrtf(ms + eps);
        for (int32_t j = 0; j < H; ++j)
            y[(size_t)i * H + j] = xi[j] * inv * oracle_half_to_float(w[j]);
    }
}

void oracle_rope(float *v, int32_t d, int32_t pos, float base)
{
    int32_t half = d / 2;
    for (int32_t t = 0; t < half; ++t) {
        double theta = pow((double)base, -2.0 * (double)t / (double)d);
        double ang = (double)pos * theta;
        float c = (float)cos(ang);
        float s = (float)sin(ang);
        float a = v[t];
        float b = v[t + half];
        v[t]        = a * c - b * s;
        v[t + half] = a * s + b * c;
    }
}

static int32_t slot_of(const oracle_seqs *sq, int32_t b)
{
    return sq->slots ? sq->slots[b] : b;
}

void oracle_rope_append(float *qkv, const oracle_dims *dm, float *kcache, float *vcache,
                        const oracle_seqs *sq, int32_t n)
{
    int32_t h = dm->n_heads, g = dm->n_kv_heads, d = dm->head_dim;
    int32_t width = (h + 2 * g) * d;
    int32_t row = 0;
    (void)n;
    for (int32_t b = 0; b < sq->B; ++b) {
        int32_t slot = slot_of(sq, b);
        for (int32_t i = 0; i < sq->q_lens[b]; ++i, ++row) {
            int32_t pos = sq->kv_lens[b] - sq->q_lens[b] + i;
            float *qrow = qkv + (size_t)row * width;
            float *krow = qrow + (size_t)h * d;
            float *vrow = krow + (size_t)g * d;
            for (int32_t j = 0; j < h; ++j)
                oracle_rope(qrow + (size_t)j * d, d, pos, dm->rope_base);
            for (int32_t j = 0; j < g; ++j)
                oracle_rope(krow + (size_t)j * d, d, pos, dm->rope_base);
            size_t at = ((size_t)slot * dm->kv_capacity + (size_t)pos) * (size_t)(g * d);
            memcpy(kcache + at, krow, sizeof(float) * (size_t)(g * d));
            memcpy(vcache + at, vrow, sizeof(float) * (size_t)(g * d));
        }
    }
}

void oracle_attention(const float *q, const float *kcache, const float *vcache,
                      const oracle_dims *dm, const oracle_seqs *sq,
                      float *out, int32_t n, float *probs)
{
    int32_t h = dm->n_heads, g = dm->n_kv_heads, d = dm->head_dim;
    int32_t cap = dm->kv_capacity;
    int32_t rep = h / g;
    /* row -> (sequence, position) table */
    int32_t *row_slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    int32_t *row_pos  = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n > 0 ? n : 1));
    int32_t row = 0;
    for (int32_t b = 0; b < sq->B; ++b)
        for (int32_t i = 0; i < sq->q_lens[b]; ++i, ++row) {
            row_slot[row] = slot_of(sq, b);
            row_pos[row]  = sq->kv_lens[b] - sq->q_lens[b] + i;
        }
    float inv_sqrt_d = 1.0f / sqrtf((float)d);

#pragma omp parallel
    {
        float *s = (float *)malloc(sizeof(float) * (size_t)cap);
#pragma omp for schedule(dynamic, 1) collapse(2)
        for (int32_t i = 0; i < n; ++i) {
            for (int32_t j = 0; j < h; ++j) {
                int32_t pos = row_pos[i];
                int32_t kvh = j / rep;
                const float *qv = q + ((size_t)i * h + j) * d;
                const float *Kb = kcache + (size_t)row_slot[i] * cap * (size_t)(g * d);
                const float *Vb = vcache + (size_t)row_slot[i] * cap * (size_t)(g * d);
                float smax = -INFINITY;
                for (int32_t t = 0; t <= pos; ++t) {
                    const float *kv = Kb + ((size_t)t * g + kvh) * d;
                    float dot = 0.0f;
                    for (int32_t e = 0; e < d; ++e)
                        dot += qv[e] * kv[e];
                    s[t] = dot * inv_sqrt_d;
                    if (s[t] > smax) smax = s[t];
                }
                float denom = 0.0f;
                for (int32_t t = 0; t <= pos; ++t) {
                    s[t] = expf(s[t] - smax);
                    denom += s[t];
                }
                for (int32_t t = 0; t <= pos; ++t)
                    s[t] = s[t] / denom;
                /* o[e] = sum_{t ascending} p_t V[t][e] for every e */
                float *o = out + ((size_t)i * h + j) * d;
                for (int32_t e = 0; e < d; ++e)
                    o[e] = 0.0f;
                for (int32_t t = 0; t <= pos; ++t) {
                    const float *vv = Vb + ((size_t)t * g + kvh) * d;
                    for (int32_t e = 0; e < d; ++e)
                        o[e] += s[t] * vv[e];
                }
                if (probs)
                    memcpy(probs + ((size_t)i * h + j) * cap, s, sizeof(float) * (size_t)(pos + 1));
            }
        }
        free(s);
    }
    free(row_slot);
    free(row_pos);
}

void oracle_swiglu(const float *gu, float *a, int32_t n, int32_t F)
{
    for (int32_t i = 0; i < n; ++i)
        for (int32_t f = 0; f < F; ++f) {
            float gate = gu[(size_t)i * 2 * F + f];
            float up   = gu[(size_t)i * 2 * F + F + f];
            a[(size_t)i * F + f] = gate / (1.0f + expf(-gate)) * up;
        }
}

static int descriptor_ok(const oracle_dims *dm, const oracle_layer_weights *w,
                         const oracle_seqs *sq, int32_t n)
{
    if (n < 1 || sq->B < 1) return 0;
    if (dm->n_kv_heads < 1 || dm->n_heads % dm->n_kv_heads != 0) return 0;
    if (dm->head_dim % 2 != 0) return 0;
    if (w->wqkv.k % 8 || w->wo.k % 8 || w->wgu.k % 8 || w->wdown.k % 8) return 0;
    int64_t total = 0;
    for (int32_t b = 0; b < sq->B; ++b) {
        if (sq->q_lens[b] < 1) return 0;
        if (sq->kv_lens[b] < sq->q_lens[b]) return 0;
        if (sq->kv_lens[b] > dm->kv_capacity) return 0;
        total += sq->q_lens[b];
    }
    return total == n;
}

int32_t oracle_decoder_layer_f32(const oracle_dims *dm, const oracle_layer_weights *w,
                                 const float *x, float *kcache, float *vcache,
                                 const oracle_seqs *sq, float *out, int32_t n,
                                 const oracle_layer_taps *taps)
{
    if (!descriptor_ok(dm, w, sq, n)) return -1;
    int32_t H = dm->hidden, h = dm->n_heads, g = dm->n_kv_heads, d = dm->head_dim, F = dm->ffn;
    int32_t qkvw = (h + 2 * g) * d;

    float *xn   = (float *)malloc(sizeof(float) * (size_t)n * H);
    float *qkv  = (float *)malloc(sizeof(float) * (size_t)n * qkvw);
    float *qbuf = (float *)malloc(sizeof(float) * (size_t)n * h * d);
    float *attn = (float *)malloc(sizeof(float) * (size_t)n * h * d);
    float *proj = (float *)malloc(sizeof(float) * (size_t)n * H);
    float *x1   = (float *)malloc(sizeof(float) * (size_t)n * H);
    float *gu   = (float *)malloc(sizeof(float) * (size_t)n * 2 * F);
    float *act  = (float *)malloc(sizeof(float) * (size_t)n * F);

    /* attention block */
    oracle_rmsnorm(x, w->norm_attn, xn, n, H, dm->rms_eps);
    oracle_dequant_matmul_g(xn, w->wqkv.q, w->wqkv.s, w->wqkv.m, w->wqkv.k, w->wqkv.group, qkv, n);
    oracle_rope_append(qkv, dm, kcache, vcache, sq, n);
    for (int32_t i = 0; i < n; ++i)
        memcpy(qbuf + (size_t)i * h * d, qkv + (size_t)i * qkvw, sizeof(float) * (size_t)(h * d));
    oracle_attention(qbuf, kcache, vcache, dm, sq, attn, n, NULL);
    oracle_dequant_matmul_g(attn, w->wo.q, w->wo.s, w->wo.m, w->wo.k, w->wo.group, proj, n);
    for (size_t e = 0; e < (size_t)n * H; ++e)
        x1[e] = x[e] + proj[e];

    /* feed-forward block */
    if (taps && taps->xn) memcpy(taps->xn, xn, sizeof(float) * (size_t)n * H);
    oracle_rmsnorm(x1, w->norm_ffn, xn, n, H, dm->rms_eps);
    oracle_dequant_matmul_g(xn, w->wgu.q, w->wgu.s, w->wgu.m, w->wgu.k, w->wgu.group, gu, n);
    oracle_swiglu(gu, act, n, F);
    oracle_dequant_matmul_g(act, w->wdown.q, w->wdown.s, w->wdown.m, w->wdown.k, w->wdown.group, proj, n);
    for (size_t e = 0; e < (size_t)n * H; ++e)
        out[e] = x1[e] + proj[e];

    if (taps) {
        if (taps->qkv)  memcpy(taps->qkv,  qkv,  sizeof(float) * (size_t)n * qkvw);
        if (taps->attn) memcpy(taps->attn, attn, sizeof(float) * (size_t)n * h * d);
        if (taps->x1)   memcpy(taps->x1,   x1,   sizeof(float) * (size_t)n * H);
        if (taps->act)  memcpy(taps->act,  act,  sizeof(float) * (size_t)n * F);
    }
    free(xn); free(qkv); free(qbuf); free(attn); free(proj); free(x1); free(gu); free(act);
    return 0;
}

int32_t oracle_decoder_layer(const oracle_dims *dm, const oracle_layer_weights *w,
                             const uint16_t *x, float *kcache, float *vcache,
                             const oracle_seqs *sq, float *out, int32_t n,
                             const oracle_layer_taps *taps)
{
    if (n < 1) return -1;
    size_t count = (size_t)n * dm->hidden;
    float *xf = (float *)malloc(sizeof(float) * count);
    for (size_t e = 0; e < count; ++e)
        xf[e] = oracle_half_to_float(x[e]);
    int32_t rc = oracle_decoder_layer_f32(dm, w, xf, kcache, vcache, sq, out, n, taps);
    free(xf);
    return rc;
}

void oracle_argmax(const float *logits, int32_t rows, int32_t V, int32_t *ids)
{
    for (int32_t i = 0; i < rows; ++i) {
        int32_t best = 0;
        for (int32_t c = 1; c < V; ++c)
            if (logits[(size_t)i * V + c] > logits[(size_t)i * V + best])
                best = c;
        ids[i] = best;
    }
}
