/*
 * relax_oracle.h -- plain CPU reference ("oracle") for one Llama-style decoder
 * layer with group-quantised int4 weights and runtime (symbolic) n / L.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the
 * smoke check and the benchmark's cpu_baseline leg may call it.  It shares no
 * code, header, table or constant with the HIP path and is written straight
 * from the definitions: scalar loops, fp32 arithmetic in ascending index order,
 * no blocking, no fusion, no reordering.  OpenMP, when enabled, only spreads
 * independent outputs (matrix rows, (row, head) pairs) over threads; the
 * arithmetic of any single output is the same sequential loop.
 *
 * What the paper fixes about this path (Relax, arXiv 2311.02103): callee
 * writes into caller-provided outputs (Sec. 3.3, destination-passing style);
 * the symbolic dims n and L arrive as ordinary runtime integers (Sec. 3.3,
 * call_tir's extra symbolic arguments; Sec. 4.1 "extra parameter s"); the
 * 4-bit weight decode is fused into the consuming matmul (Sec. 4.2, Fig. 9
 * decode_q4 case study); attention is one fused operator over a KV cache of
 * symbolic length (Sec. 4.2, custom attention pattern).  The paper prints no
 * numeric definition for any of these; the definitions below are the standard
 * Llama layer with the quantised format fixed by the workload description
 * (symmetric int4, group 32 along k, fp16 scales, 8 nibbles per uint32).
 *
 * Conventions
 *   - all pointers are host pointers;
 *   - fp16 inputs are passed as their 16-bit patterns (uint16_t) and widened
 *     exactly; every intermediate and every output is fp32;
 *   - the KV cache of the oracle is fp32, layout [slot][capacity][g][d];
 *   - L_b (kv_lens[b]) is the length of sequence b AFTER this call's tokens
 *     are appended; rows of one sequence are contiguous and in order, row i of
 *     sequence b sits at position  pos = L_b - q_len_b + i.
 */
#ifndef RELAX_ORACLE_H
#define RELAX_ORACLE_H

#include <stdint.h>
#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* IEEE binary16 bit pattern -> float, exact (subnormals, inf, nan included). */
float oracle_half_to_float(uint16_t bits);

/* Step 1: nibble c%8 of word qweight[r*(k/8)+c/8] sits in bits 4*(c%8)..+3;
 * code u in 0..15 means the integer u-8.  out[r*k+c] in -8..7.  k%8==0.     */
void oracle_unpack_int4(const uint32_t *qweight, int32_t m, int32_t k, int8_t *out);

/* Step 2: W[r,c] = (float)(u-8) * (float)scales[r*ceil(k/32) + c/32].
 * The last group of a row is short when k%32 != 0.                          */
void oracle_dequantize(const uint32_t *qweight, const uint16_t *scales,
                       int32_t m, int32_t k, float *out /* [m,k] */);

/* Step 3: out[i,r] = sum_{c ascending} x[i,c] * W[r,c], fp32.               */
void oracle_dequant_matmul(const float *x /* [n,k] */, const uint32_t *qweight,
                           const uint16_t *scales, int32_t m, int32_t k,
                           float *out /* [n,m] */, int32_t n);

/* Steps 2 and 3 for any quantisation group along k (the workload description
 * fixes 32; deployments of the paper's 4-bit models also use wider groups):
 * W[r,c] = (float)(u-8) * (float)scales[r*ceil(k/group) + c/group], the last
 * group of a row short when group does not divide k.  group <= 0 reads as 32;
 * the two functions above are these with group = 32.                        */
void oracle_dequantize_g(const uint32_t *qweight, const uint16_t *scales,
                         int32_t m, int32_t k, int32_t group, float *out /* [m,k] */);
void oracle_dequant_matmul_g(const float *x /* [n,k] */, const uint32_t *qweight,
                             const uint16_t *scales, int32_t m, int32_t k, int32_t group,
                             float *out /* [n,m] */, int32_t n);

/* Dense fp16 weight matmul (LM head): out[i,r] = sum_c x[i,c]*(float)w[r,c]. */
void oracle_half_matmul(const float *x /* [n,k] */, const uint16_t *w /* [m,k] */,
                        int32_t m, int32_t k, float *out /* [n,m] */, int32_t n);

/* RMSNorm: ms = (1/H) sum_j x_j^2 ; y_j = x_j * (1/sqrtf(ms+eps)) * w_j.     */
void oracle_rmsnorm(const float *x /* [n,H] */, const uint16_t *w /* [H] fp16 */,
                    float *y /* [n,H] */, int32_t n, int32_t H, float eps);

/* Rotary embedding of one head vector v[d] in place, half-split pairing:
 * for t < d/2, theta_t = base^(-2t/d), (a,b) = (v[t], v[t+d/2]) ->
 * (a cos(pos theta_t) - b sin(pos theta_t), a sin(pos theta_t) + b cos(...)).
 * Angle, cos and sin in double, rounded to fp32, products in fp32.          */
void oracle_rope(float *v, int32_t d, int32_t pos, float base);

typedef struct {
    int32_t B;               /* sequences in the call                        */
    const int32_t *q_lens;   /* [B] rows of each sequence, sum = n           */
    const int32_t *kv_lens;  /* [B] L_b after this call's append             */
    const int32_t *slots;    /* [B] cache slot of each sequence, NULL: b     */
} oracle_seqs;

typedef struct {
    int32_t hidden, n_heads, n_kv_heads, head_dim, ffn;
    float rms_eps, rope_base;
    int32_t kv_capacity;
} oracle_dims;

/* RoPE on the q and k parts of qkv[n,(h+2g)d] (row layout [q | k | v]) in
 * place, then K[slot][pos] = rope(k), V[slot][pos] = v.                     */
void oracle_rope_append(float *qkv, const oracle_dims *dm, float *kcache, float *vcache,
                        const oracle_seqs *sq, int32_t n);

/* Causal attention.  q[n,h,d]; row i, head j uses KV head j/(h/g); scores
 * s_t = (q . K[t]) / sqrtf(d) for 0 <= t <= pos only (nothing beyond pos is
 * read); p = softmax with max subtraction; o = sum_t p_t V[t].
 * probs, if non-NULL, receives p for every (row, head) as [n,h,kv_capacity]
 * with entries beyond pos left untouched.                                   */
void oracle_attention(const float *q, const float *kcache, const float *vcache,
                      const oracle_dims *dm, const oracle_seqs *sq,
                      float *out /* [n,h,d] */, int32_t n, float *probs);

/* a[i,f] = silu(gu[i,f]) * gu[i,F+f], silu(z) = z / (1 + expf(-z)).          */
void oracle_swiglu(const float *gu /* [n,2F] */, float *a /* [n,F] */, int32_t n, int32_t F);

typedef struct {
    const uint32_t *q;   /* [m, k/8]           */
    const uint16_t *s;   /* [m, ceil(k/group)] */
    int32_t m, k;
    int32_t group;       /* columns per scale; <= 0 reads as 32 */
} oracle_qmat;

typedef struct {
    oracle_qmat wqkv;    /* rows [Wq (h d) ; Wk (g d) ; Wv (g d)], k = H     */
    oracle_qmat wo;      /* [H, h d]                                         */
    oracle_qmat wgu;     /* rows [gate (F) ; up (F)], k = H                  */
    oracle_qmat wdown;   /* [H, F]                                           */
    const uint16_t *norm_attn, *norm_ffn;   /* [H] fp16                      */
} oracle_layer_weights;

/* Optional taps on the layer's intermediates (any may be NULL).             */
typedef struct {
    float *xn;     /* [n,H]         RMSNorm(x)                               */
    float *qkv;    /* [n,(h+2g)d]   after RoPE                               */
    float *attn;   /* [n,h d]                                                */
    float *x1;     /* [n,H]         x + attn Wo^T                            */
    float *act;    /* [n,F]         SwiGLU output                            */
} oracle_layer_taps;

/* The whole layer: RMSNorm -> QKV -> RoPE + append -> attention -> O-proj +
 * residual -> RMSNorm -> gate/up -> SwiGLU -> down + residual.
 * x: fp16 bit patterns [n,H]; out: fp32 [n,H]; caches fp32, updated.
 * Returns 0, or -1 on an inconsistent descriptor (sum q_lens != n, L < q_len,
 * L > capacity, h % g != 0, odd d, k % 8 != 0).                             */
int32_t oracle_decoder_layer(const oracle_dims *dm, const oracle_layer_weights *w,
                             const uint16_t *x, float *kcache, float *vcache,
                             const oracle_seqs *sq, float *out, int32_t n,
                             const oracle_layer_taps *taps);

/* Same layer, residual stream kept in fp32 from call to call (model stack). */
int32_t oracle_decoder_layer_f32(const oracle_dims *dm, const oracle_layer_weights *w,
                                 const float *x, float *kcache, float *vcache,
                                 const oracle_seqs *sq, float *out, int32_t n,
                                 const oracle_layer_taps *taps);

/* Greedy pick: lowest index among the maxima of each row of logits[rows,V]. */
void oracle_argmax(const float *logits, int32_t rows, int32_t V, int32_t *ids);

int32_t oracle_num_threads(void);

#ifdef __cplusplus
}
#endif
#endif
