/*
 * relax_mi355.h -- C ABI of the MI355X (gfx950) implementation of the
 * dynamic-shape int4 Llama-style decoder layer behind the LLM results of
 * "Relax: Composable Abstractions for End-to-End Dynamic Machine Learning"
 * (arXiv 2311.02103).
 *
 * Calling rules, each taken from the paper's statement of the problem:
 *   - Destination-passing style (Sec. 3.3): the caller owns and passes every
 *     output, the KV cache and the workspace; the library allocates nothing
 *     and keeps no hidden state between calls.
 *   - Symbolic dimensions are ordinary runtime integers passed next to the
 *     tensors (Sec. 3.3, the extra symbolic arguments of call_tir; Sec. 4.1,
 *     the extra parameter bound to n).  n (rows in the call), L (KV length)
 *     and B (sequences) may change on every call; ONE compiled library serves
 *     every value -- nothing is specialised, rebuilt or cached per shape
 *     (Sec. 5.1: compiled once for arbitrary batch size and sequence length).
 *     Only the static model dimensions in relax_layer_dims are treated as
 *     constants of a model (Sec. 3.3: specialise static dims, keep n dynamic).
 *   - Scratch memory of the kernels (split-L attention partials, staging) is
 *     lifted to one caller-provided workspace sized from upper bounds on the
 *     symbolic dims (Sec. 4.3 upper-bound planning, Sec. 4.4 workspace
 *     lifting): relax_workspace_bytes(dims, n_max, L_max, B_max).
 *   - Shape constraints are checked at the function boundary and reported as
 *     error codes (Sec. 3.2 match_cast runtime checks, Sec. 4.1 boundary
 *     checks).  All checks run on the host BEFORE anything is enqueued: a call
 *     that returns an error has written nothing.
 *   - The int4 decode never materialises a dense weight matrix: it is fused
 *     into the consuming matmul (Sec. 4.2, decode_q4 case study); a matrix-
 *     vector kernel serves small n, an MFMA GEMM serves large n, chosen from
 *     the runtime value of n inside the same entry point (Sec. 5.1).
 *
 * Memory spaces: every pointer is a DEVICE pointer unless its comment says
 * "host".  fp16 tensors are passed as uint16_t bit patterns.  All work is
 * enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream)
 * and is asynchronous; the return value reports validation / launch errors.
 *
 * Storage format of a quantised matrix W[m,k] (k % 8 == 0) with quantisation group G
 * (32 unless the descriptor says 64 or 128):
 *   q : uint32 [m, k/8]        element c of row r is nibble c%8 (bits
 *                              4*(c%8)..+3) of word q[r*(k/8) + c/8];
 *                              code u in 0..15 stands for the integer u-8
 *   s : fp16   [m, ceil(k/G)]  one scale per G consecutive c (last group
 *                              short when k % G != 0)
 *   W[r,c] = (u - 8) * s[r, c/G]
 */
#ifndef RELAX_MI355_H
#define RELAX_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t relax_status;
enum {
    RELAX_OK              =  0,
    RELAX_ERR_NULL        = -1,   /* a required pointer is NULL                          */
    RELAX_ERR_SHAPE       = -2,   /* n<1, k%8!=0, sum(q_lens)!=n, L_b<q_len_b, h%g!=0... */
    RELAX_ERR_CAPACITY    = -3,   /* L_b > kv_capacity, slot out of range                */
    RELAX_ERR_WORKSPACE   = -4,   /* ws_bytes below relax_workspace_bytes(...), ws not 256-byte aligned */
    RELAX_ERR_UNSUPPORTED = -5,   /* head_dim not in {64,128}, group not in {32,64,128}, k too large */
    RELAX_ERR_HIP         = -6    /* the HIP runtime reported a launch error             */
};

typedef void *relax_stream;       /* hipStream_t */

/* Static dimensions of a layer (constants of a model, not symbolic).                    */
typedef struct {
    int32_t hidden;               /* H                                                   */
    int32_t n_heads;              /* h  query heads                                      */
    int32_t n_kv_heads;           /* g  KV heads, h % g == 0                             */
    int32_t head_dim;             /* d  in {64, 128}                                     */
    int32_t ffn;                  /* F                                                   */
    int32_t group;                /* quantisation group of the four matrices: 32, 64 or 128 */
    float   rms_eps;
    float   rope_base;
    int32_t kv_capacity;          /* L_cap: positions per cache slot                     */
    int32_t kv_slots;             /* number of cache slots                               */
} relax_layer_dims;

/* A quantised matrix in the storage format described at the top.                        */
typedef struct {
    const uint32_t *q;            /* [m, k/8]                                            */
    const uint16_t *s;            /* [m, ceil(k/group)] fp16                             */
    int32_t m, k;
    int32_t group;                /* columns per scale: 32, 64 or 128 (0 reads as 32; the 4-bit deployments of
                                     Sec. 5.3 come in several group sizes).  Inside a layer every matrix must carry
                                     the group of relax_layer_dims.  Other values: RELAX_ERR_UNSUPPORTED.  The 3-bit
                                     calls ignore the field (their group is 32).                                 */
} relax_qmat;

typedef struct {
    relax_qmat wqkv;              /* rows [Wq (h*d) ; Wk (g*d) ; Wv (g*d)], k = H        */
    relax_qmat wo;                /* [H, h*d]                                            */
    relax_qmat wgu;               /* rows [gate (F) ; up (F)], k = H                     */
    relax_qmat wdown;             /* [H, F]                                              */
    const uint16_t *norm_attn;    /* [H] fp16                                            */
    const uint16_t *norm_ffn;     /* [H] fp16                                            */
} relax_layer_weights;

/* KV cache of one layer.  K holds keys AFTER rotary embedding.                          */
typedef struct {
    uint16_t *k;                  /* [kv_slots, kv_capacity, g, d] fp16                  */
    uint16_t *v;                  /* [kv_slots, kv_capacity, g, d] fp16                  */
    const float *rope;            /* [kv_capacity, d/2, 2] (cos, sin) of pos*base^(-2t/d),
                                     filled once by relax_rope_table_init                */
} relax_kv_cache;

/* The ragged batch of one call.  Rows of a sequence are contiguous and in order; row i
 * of sequence b sits at position kv_lens[b] - q_lens[b] + i.  A prefill of one sequence
 * is (B=1, {n}, {L}); a batched decode step is (B=n, {1,...}, {L_b}).  Up to 16 sequences ride in kernel arguments;
 * a longer descriptor without device_table is written to a table at the front of the workspace by small kernels on
 * the call's stream (32 sequences per launch, carried in their arguments): the host arrays are not needed after the
 * call returns, the host never waits, and the call can be captured in a graph.                                  */
typedef struct {
    int32_t B;
    const int32_t *q_lens;        /* host [B], each >= 1, sum == n                       */
    const int32_t *kv_lens;       /* host [B], L_b AFTER this call's rows are appended   */
    const int32_t *slots;         /* host [B] cache slot per sequence; NULL: slot b = b  */
    const int32_t *device_table;  /* NULL, or device [4][B] int32: q_start, q_len, kv_len, slot per sequence
                                     (q_start = first row of the sequence in the call).  The device-side form
                                     of the descriptor -- the runtime shape heap of Sec. 4.7 -- for callers that
                                     capture a call in a graph and replay it (Sec. 4.5 graph offloading): when
                                     set, the kernels read positions and slots THERE, at run time, and the host
                                     arrays above only shape the launch: B, q_lens and n must be exact, kv_lens
                                     must be upper bounds of what the table will ever hold while the captured
                                     call is replayed (they size the attention plan; the capacity check is made
                                     on them), slots are ignored.  The caller owns the table, keeps it alive
                                     and consistent (kv_len >= q_len, within the bounds) and updates it between
                                     replays, e.g. with a one-thread kernel in the same graph; the call then does
                                     no host-to-device copy and no synchronisation.                          */
} relax_seqs;

/* Bytes of workspace that any call with n <= n_max, every L_b <= L_max and B <= B_max
 * needs (Sec. 4.3: static plan from upper bounds; Sec. 4.4: lifted kernel scratch).
 * Returns 0 if dims is NULL or inconsistent.                                            */
size_t relax_workspace_bytes(const relax_layer_dims *dims, int32_t n_max, int32_t L_max, int32_t B_max);

/* The memory plan behind relax_workspace_bytes (Sec. 4.3, Alg. 3: dynamic shape-aware memory planning).  The
 * intermediates of a layer call -- xn, qkv, the attention output and partials, x1, act and the workspace lifted
 * out of the few-row matmul -- are walked in program order; an allocation reuses a free storage when its size
 * provably fits for every value of the symbols (c1*n bytes into c2*n bytes when c1 <= c2; an opaque expression of
 * (n, L, B) only into the same expression), otherwise a new storage is opened; a storage returns to the pool after
 * the last use of its tensor.  The reuse structure therefore does not depend on n, L, B, every storage grows with
 * them, and the plan at upper bounds covers every smaller call.
 * relax_workspace_plan reports that plan for one (n, L, B): one entry per tensor (operations of the layer:
 * 1 QKV + rotary + append, 2 attention, 3 output projection, 4 second norm, 5 gate/up, 6 down), `offset` in bytes
 * from the start of the workspace, and the bytes of the planned region with and without reuse (every storage,
 * resp. tensor, rounded up to 256 bytes; the fixed front part of the workspace -- the flag line and the
 * descriptor table -- is in neither).  entries may be NULL (sizes only); capacity < *count: RELAX_ERR_WORKSPACE.
 * Host-only: nothing is enqueued.                                                                                */
typedef struct {
    char name[24];
    int32_t first_op, last_op;    /* the tensor is allocated in front of first_op and dead after last_op          */
    int32_t storage;              /* index of the storage it lives in; tensors with equal storage share memory    */
    int32_t pinned;               /* 1: live for the whole call and across the layers of relax_model_step (xn)    */
    uint64_t offset, bytes, storage_bytes;
} relax_plan_entry;
relax_status relax_workspace_plan(const relax_layer_dims *dims, int32_t n, int32_t L, int32_t B, relax_plan_entry *entries,
                                  int32_t capacity, int32_t *count, size_t *planned_bytes, size_t *unplanned_bytes);
/* The same query under a chosen reuse rule.  rule 1 is Alg. 3 as Sec. 4.3 states it: a free storage is reused only when
 * the symbolic size of the request is proven EQUAL to the storage's (the same multiple of n, or the same opaque
 * expression).  rule 0 is the extension the calls of this library lay their workspace out with (and what
 * relax_workspace_plan reports): the request only has to fit provably, c1*n bytes into c2*n bytes when c1 <= c2.
 * Offsets of rule 1 describe the layout that rule would give; no call uses it.  Other rules: RELAX_ERR_UNSUPPORTED. */
relax_status relax_workspace_plan_rule(const relax_layer_dims *dims, int32_t n, int32_t L, int32_t B, int32_t rule,
                                       relax_plan_entry *entries, int32_t capacity, int32_t *count, size_t *planned_bytes,
                                       size_t *unplanned_bytes);

/* The first 256 bytes of a layer or model workspace are a line of flags that kernels raise for conditions the host
 * cannot check because they are device data: bit 1 of word 0 = relax_model_step met a token id outside [0, vocab) and
 * read it as id 0.  relax_workspace_init clears the line (one small kernel on `stream`); a workspace whose flags are
 * never read needs no initialisation.  relax_workspace_error copies word 0 to the host (synchronous).
 * Every workspace pointer passed to this library must be 256-byte aligned (RELAX_ERR_WORKSPACE otherwise): the
 * intermediates inside it are read with 16-byte accesses and as MFMA operand tiles.                               */
relax_status relax_workspace_init(const relax_layer_dims *dims, void *ws, size_t ws_bytes, relax_stream stream);
relax_status relax_workspace_error(const relax_layer_dims *dims, const void *ws, int32_t *flag_host);

/* Bytes of the rotary table for these dims, and the call that fills it on the device
 * (angles, cos and sin evaluated in fp64, stored as fp32).  Pairing is half-split:
 * element t < d/2 rotates with element t + d/2 at frequency base^(-2t/d).               */
size_t       relax_rope_table_bytes(const relax_layer_dims *dims);
relax_status relax_rope_table_init(const relax_layer_dims *dims, float *table, relax_stream stream);

/* out[i,r] = sum_c x[i,c] * W[r,c] with W decoded on the fly (Sec. 4.2 fused decode;
 * Sec. 5.1: the kernel is picked from the symbolic n at run time -- matrix-vector kernel
 * for one row, split-K MFMA kernel for a few rows, tiled MFMA GEMM for many).
 * x [n,k] fp16, out [n,m] fp16, fp32 accumulation.  The few-row kernel keeps its split-K
 * partial tiles in ws (Sec. 4.4, lifted workspace): relax_matmul_workspace_bytes(w, n_max)
 * is enough for every n <= n_max; with ws == NULL or fewer bytes the call still succeeds
 * through the other two kernels.  Errors: NULL, SHAPE (n<1, m<1, k<8, k%8),
 * UNSUPPORTED (k > 28672).                                                              */
size_t       relax_matmul_workspace_bytes(const relax_qmat *w, int32_t n_max);
relax_status relax_dequant_matmul(const uint16_t *x, const relax_qmat *w, uint16_t *out, int32_t n,
                                  void *ws, size_t ws_bytes, relax_stream stream);

/* The same matmul with plain fp16 weights (the fp16-weight configurations of the paper's LLM evaluation,
 * Sec. 5.1): out[i,r] = sum_c x[i,c] * w[r,c], x [n,k] fp16, w [m,k] fp16 row-major, out [n,m] fp16, fp32
 * accumulation, dispatched on the runtime n like the int4 call: passes of up to 8 rows through the fp16
 * matrix-vector kernel (the one the LM head uses) for a few rows, the tiled MFMA GEMM without its decode
 * step (k % 128 == 0, m % 4 == 0) from the row count on at which its estimated time falls below that of the
 * passes -- 24 rows on a 4096 x 4096 matrix, 8 on 22016 x 4096 (measured: bench.py --workload half_sweep).
 * the test switch "half_matmul_gemm_rows" (relax_mi355_bench.h) with r > 0 fixes the crossover at r rows instead (0, the
 * default: by estimate).  Device pointers, x and w 16-byte aligned.  Errors: NULL, SHAPE (n<1, m<1, k<8,
 * k%8, alignment), UNSUPPORTED (k > 73728).                                                                */
relax_status relax_half_matmul(const uint16_t *x, const uint16_t *w, uint16_t *out, int32_t n, int32_t m,
                               int32_t k, relax_stream stream);

/* Two optional parts (the norm and the rotary step are separated by the QKV matmul, so
 * they cannot be one pass; either part is skipped when its first pointer is NULL):
 *  part 1  y[i,:] = x[i,:] * rsqrt(mean(x[i,:]^2) + eps) * w      x,y [n,H] fp16, w [H]
 *  part 2  rotary embedding in place on the q and k columns of qkv [n,(h+2g)d] fp16
 *          (row layout [q | k | v]) at each row's position, then K[slot][pos] = k,
 *          V[slot][pos] = v.  Needs dims, cache (with rope table) and seqs.
 * Errors: NULL, SHAPE, CAPACITY, UNSUPPORTED as listed in the enum.                     */
relax_status relax_rmsnorm_rope(const uint16_t *x, const uint16_t *w, uint16_t *y, int32_t n, int32_t H,
                                float eps, uint16_t *qkv, const relax_layer_dims *dims,
                                const relax_kv_cache *cache, const relax_seqs *seqs, relax_stream stream);

/* Causal attention over the cache (Sec. 4.2, the fused attention operator; KV length is
 * symbolic).  q [n,h,d] fp16 (already rotated), out [n,h,d] fp16.  Row i of sequence b
 * attends to cache positions 0..pos_i of its slot, which must already hold this call's
 * keys/values; nothing beyond pos_i is read.  Query head j uses KV head j / (h/g).
 * softmax scale 1/sqrt(d), fp32 softmax.  Decode rows are split along L over many
 * workgroups and merged from the workspace.                                             */
relax_status relax_attention(const uint16_t *q, const relax_kv_cache *cache, const relax_seqs *seqs,
                             const relax_layer_dims *dims, uint16_t *out, int32_t n,
                             void *ws, size_t ws_bytes, relax_stream stream);

/* relax_attention for callers that cannot allocate or bring a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, checks, kernels and results as relax_attention, without
 * ws / ws_bytes: the split-L partials live in a device array that is part of the library image (a file-scope
 * __device__ array of relax_attention_static_max_bytes() = 16 MiB; every GPU the library runs on holds its copy until
 * the process ends).  The call allocates nothing and frees nothing; its first call on a device looks the array's
 * address up once.  Limits: the partials of the call -- relax_workspace_plan's "attn_partials" entry for (n, max L_b),
 * e.g. 0.55 MB for one 7B-shaped decode row, 8.5 MB for 16 rows of the 70B shape at L = 8192 -- must fit the array
 * (RELAX_ERR_WORKSPACE otherwise), and a descriptor without device_table may hold at most 16 sequences
 * (RELAX_ERR_UNSUPPORTED: copying a longer one to the device needs a workspace).  All calls on one GPU share the array,
 * which keeps the previous call's contents (every partial a call reads it has written itself, nothing needs clearing):
 * calls that overlap on one GPU -- different streams, or graphs replayed concurrently -- race; calls on one stream
 * are ordered and safe.                                                                                          */
size_t       relax_attention_static_max_bytes(void);
relax_status relax_attention_static(const uint16_t *q, const relax_kv_cache *cache, const relax_seqs *seqs,
                                    const relax_layer_dims *dims, uint16_t *out, int32_t n, relax_stream stream);

/* The whole layer on n rows:
 *   xn = RMSNorm(x; norm_attn); qkv = xn Wqkv^T; rotary(q,k); append k,v;
 *   a = attention(q); x1 = x + a Wo^T;
 *   gu = RMSNorm(x1; norm_ffn) Wgu^T; act = silu(gate) * up; out = x1 + act Wdown^T
 * x, out [n,H] fp16 (out may alias x).  The cache is updated at positions
 * kv_lens[b]-q_lens[b] .. kv_lens[b]-1 of each sequence's slot.                         */
relax_status relax_decoder_layer(const relax_layer_dims *dims, const relax_layer_weights *weights,
                                 const uint16_t *x, const relax_kv_cache *cache, const relax_seqs *seqs,
                                 uint16_t *out, int32_t n, void *ws, size_t ws_bytes, relax_stream stream);

/* A stack of decoder layers with its embedding and output head (the end-to-end LLM of
 * Sec. 5.1: the layer above repeated, between a token-embedding gather and a final
 * RMSNorm + unquantised fp16 vocabulary projection).  `layers` is a HOST array of
 * n_layers weight structs (their pointers are device pointers); embedding and lm_head
 * are device fp16 [vocab, hidden], norm_final device fp16 [hidden].  n_layers may be 0. */
typedef struct {
    relax_layer_dims dims;
    int32_t n_layers, vocab;
    const relax_layer_weights *layers;
    const uint16_t *embedding;
    const uint16_t *norm_final;
    const uint16_t *lm_head;
} relax_model;

/* Bytes of workspace for relax_model_step over every call with n <= n_max rows,
 * B <= B_max sequences, kv_lens <= L_max: the layer workspace (shared by all layers,
 * which run one after another), two [n_max, hidden] fp16 activation buffers, the
 * normalised last rows and [B_max, vocab] fp16 logits.  Its first 256 bytes are the flag
 * line described at relax_workspace_init (clear it once if the flags are read).
 * Returns 0 for invalid arguments.                                                      */
size_t relax_model_workspace_bytes(const relax_model *model, int32_t n_max, int32_t L_max, int32_t B_max);

/* One step of the whole model on n rows (prefill, decode or a ragged mix, as described
 * by seqs):  x = E[ids];  x = layer_l(x) for l = 0..n_layers-1, layer l using caches[l]
 * (a HOST array of n_layers cache structs with the dims' capacity and slots);
 * y_b = RMSNorm(x[last row of sequence b]; norm_final);  logits[b,:] = y_b lm_head^T
 * (fp32 accumulation, stored fp16);  next_ids[b] = lowest index among the maxima of
 * logits[b,:] as stored (greedy decoding, the paper's generation protocol).
 * ids: device int32 [n].  logits: device fp16 [B, vocab] or NULL (then they stay in the
 * workspace).  next_ids: device int32 [B] or NULL.  An id outside [0, vocab) is read as
 * id 0 and raises bit 1 of the flag relax_workspace_error reports.
 * Errors as relax_decoder_layer; hidden must be a multiple of 8.                        */
relax_status relax_model_step(const relax_model *model, const int32_t *ids, const relax_kv_cache *caches,
                              const relax_seqs *seqs, uint16_t *logits, int32_t *next_ids, int32_t n,
                              void *ws, size_t ws_bytes, relax_stream stream);

/* Test exports for the bit-exactness requirement on decoding and indexing: the device
 * decode of (word, nibble, scale group) written out densely, one element per thread.
 * relax_unpack_int4: out int8 [m,k] in -8..7.  relax_dequantize: out fp32 [m,k].        */
relax_status relax_unpack_int4(const relax_qmat *w, int8_t *out, relax_stream stream);
relax_status relax_dequantize(const relax_qmat *w, float *out, relax_stream stream);

/* 3-bit weights (Sec. 5.3: 3-bit quantised models are what fits the smaller devices; the
 * paper prints no bit layout, this one mirrors the 4-bit format).  A relax_qmat whose q is
 * uint32 [m][3k/32] and whose s is fp16 [m][k/32], both device memory, row-major: a group
 * of 32 columns shares one scale, its 32 codes u in 0..7 lie end to end, 3 bits each, in
 * three little-endian words (code c at bits 3c..3c+2 of the 96-bit string), and the weight
 * is (u - 4) * scale.  k % 32 == 0.
 * relax_unpack_q3: out int8 [m,k] in -4..3 (device), bit-exact decode export.
 * relax_dequant_matmul_q3: out[n,m] fp16 = x[n,k] fp16 (device, 16-byte aligned) times the
 * decoded matrix, fp32 accumulation; a matrix-vector kernel run once per row of x (meant for
 * decode-sized n; every row of x streams the matrix again), k <= 12288 (longer rows:
 * RELAX_ERR_UNSUPPORTED), n <= 65535.  Asynchronous on `stream`; nothing is allocated and
 * nothing is owned.  NULL pointers: RELAX_ERR_NULL; bad sizes or alignment: RELAX_ERR_SHAPE. */
relax_status relax_unpack_q3(const relax_qmat *w, int8_t *out, relax_stream stream);
relax_status relax_dequant_matmul_q3(const uint16_t *x, const relax_qmat *w, uint16_t *out, int32_t n, relax_stream stream);

/* The GPU-native 3-bit layout: the same bits per group in an order the kernels decode at a third of the cost (one
 * vector operation yields a ready fp16 pair); with it a 3-bit matrix-vector product takes the time of the 4-bit one
 * on the same shape (from the canonical stream it was a third slower).  Per group of 32 columns (codes u_0..u_31) and its three words: position j (0..4) of word w holds
 * u_{2(5w+j)} in bits 3j..3j+2 and u_{2(5w+j)+1} in bits 16+3j..16+3j+2; bit i of u_30 is bit 15 of word i, bit i of
 * u_31 is bit 31 of word i.  Scales are unchanged.
 * relax_repack_q3: canonical q (as above) -> native_q, device uint32 [m][3k/32] owned by the caller, not in place; a
 * one-time step at load time (Sec. 4.6: weights are prepared once for the kernels that serve them).
 * relax_unpack_q3_native: out int8 [m,k] in -4..3 from a native matrix -- equals relax_unpack_q3 of the canonical one.
 * relax_dequant_matmul_q3_native: out[n,m] fp16 = x[n,k] times the decoded native matrix, fp32 accumulation.  Up to 15
 * rows of x are taken 4, 2 or 1 per pass over the matrix (k <= 4096: 4; k <= 8192: 2), the decode of a weight shared
 * by the rows of a pass, so a few rows cost little more than one (k <= 12288).  From 16 rows on, a matrix with
 * k % 128 == 0 and m % 4 == 0 (out 8-byte aligned) goes through the tiled MFMA GEMM that serves the 4-bit format at
 * large n, its decode step replaced by the 3-bit one: the matrix is read once whatever n is, and k is not limited.
 * x 16-byte aligned; errors as the canonical call. */
relax_status relax_repack_q3(const relax_qmat *canonical, uint32_t *native_q, relax_stream stream);
relax_status relax_unpack_q3_native(const relax_qmat *w, int8_t *out, relax_stream stream);
relax_status relax_dequant_matmul_q3_native(const uint16_t *x, const relax_qmat *w, uint16_t *out, int32_t n, relax_stream stream);

/* The whole layer on 3-bit weights (Sec. 5.3: the 3-bit models are what the paper deploys where memory is short): the
 * same computation as relax_decoder_layer, same dims, cache, descriptor and x / out conventions, with the four matrices of
 * `weights` in the GPU-native 3-bit layout above (group 0 or 32; their rows within what the 3-bit matmul takes: k % 32 == 0,
 * k <= 12288).  One row (n == 1) runs the five fused launches of the 4-bit decode layer on the 3-bit stream of the same
 * matrix-vector kernel (norms, rotary + append, attention merge, residuals and SwiGLU inside the four launches, fp32 sums
 * not rounded in between).  From two rows on the 3-bit matmuls have the plain fp16 epilogue only, so the layer is a sequence of launches of their own
 * -- RMSNorm, matmul, rotary + append, attention, matmul, residual add, RMSNorm, matmul, SwiGLU, matmul, residual add --
 * with the dispatch on n of relax_dequant_matmul_q3_native inside (matrix-vector passes below 16 rows, tiled MFMA GEMM from
 * there on); nothing is fused, a 3-bit matmul output is rounded to fp16 before the residual is added, the residual stream
 * x1 stays fp32 between the two halves of the layer.  Its workspace is its own: relax_layer_q3_workspace_bytes(dims, n_max,
 * L_max, B_max) bytes, 256-byte aligned (0 for invalid arguments); the first 256 bytes are the flag line of
 * relax_workspace_init, which this call neither reads nor writes.  hidden % 8 == 0, ffn % 8 == 0, x and out 16-byte
 * aligned.  Asynchronous on `stream`; allocates nothing; errors as relax_decoder_layer, checked before anything is enqueued. */
size_t       relax_layer_q3_workspace_bytes(const relax_layer_dims *dims, int32_t n_max, int32_t L_max, int32_t B_max);
relax_status relax_decoder_layer_q3(const relax_layer_dims *dims, const relax_layer_weights *weights, const uint16_t *x,
                                    const relax_kv_cache *cache, const relax_seqs *seqs, uint16_t *out, int32_t n, void *ws,
                                    size_t ws_bytes, relax_stream stream);

/* The whole layer on plain fp16 weights (the fp16 models of the paper's LLM evaluation, Sec. 5.1): the same computation,
 * dims, cache, descriptor and x / out conventions as relax_decoder_layer, the four matrices row-major fp16 -- wqkv
 * [(h + 2g) d, H], wo [H, h d], wgu [2F, H] (gate rows, then up rows), wdown [H, F] -- and the two norm vectors, all device
 * memory, 16-byte aligned, owned by the caller.  From two rows on it is, like the 3-bit layer, a sequence of launches of
 * their own around relax_half_matmul's dispatch on n (matrix-vector passes for a few rows, tiled MFMA GEMM from the row
 * count on at which its estimate is lower): nothing is fused, a matmul output is rounded to fp16 before the residual is
 * added, x1 stays fp32.  One row (n == 1, rows of at most 12288 columns) runs the five fused launches of the 4-bit decode
 * layer on the fp16 stream of the same matrix-vector kernel: the norms, rotary + append, the attention merge, the
 * residuals and SwiGLU happen inside the four matrix-vector launches, on fp32 sums that are not rounded in between.
 * Workspace: relax_layer_f16_workspace_bytes(dims, n_max, L_max, B_max) bytes, 256-byte aligned (0 for invalid arguments).
 * hidden % 8 == 0, ffn % 8 == 0, rows of at most 73728 columns.  Asynchronous on `stream`; allocates nothing; errors as
 * relax_decoder_layer, checked before anything is enqueued.                                                         */
typedef struct {
    const uint16_t *wqkv, *wo, *wgu, *wdown;
    const uint16_t *norm_attn, *norm_ffn;
} relax_layer_f16_weights;
size_t       relax_layer_f16_workspace_bytes(const relax_layer_dims *dims, int32_t n_max, int32_t L_max, int32_t B_max);
relax_status relax_decoder_layer_f16(const relax_layer_dims *dims, const relax_layer_f16_weights *weights, const uint16_t *x,
                                     const relax_kv_cache *cache, const relax_seqs *seqs, uint16_t *out, int32_t n, void *ws,
                                     size_t ws_bytes, relax_stream stream);

/* Build identity of the loaded binary (one binary serves every shape).                  */
const char *relax_build_id(void);

#ifdef __cplusplus
}
#endif
#endif
