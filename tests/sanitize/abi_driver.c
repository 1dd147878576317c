/* Drives the host side of the C ABI -- the argument checks and the workspace planner, everything a call does before it
 * enqueues anything -- against a build of the library whose host code is compiled with -fsanitize=address,undefined
 * (tests/test_sanitizers.py).  No GPU is needed: every call here returns on the host.  Device pointers are fake but
 * aligned addresses that the host code must never dereference; host arrays (sequence descriptors, plan entries) are
 * malloc'ed at their exact size so that a read or write past them lands in a red zone. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "relax_mi355.h"
#include "relax_mi355_bench.h"

static int failures = 0;
#define EXPECT(call, want) do { relax_status got_ = (call); if (got_ != (want)) { \
    fprintf(stderr, "%s:%d: %s returned %d, expected %d\n", __FILE__, __LINE__, #call, (int)got_, (int)(want)); ++failures; } } while (0)
#define EXPECT_TRUE(cond) do { if (!(cond)) { fprintf(stderr, "%s:%d: %s is false\n", __FILE__, __LINE__, #cond); ++failures; } } while (0)

#define DEV ((void *)(uintptr_t)0x7f0000100000ull)      /* a plausible, 256-byte aligned device address, never read */

static int32_t *ints(int count, int32_t value)
{
    int32_t *p = malloc((size_t)(count ? count : 1) * sizeof(int32_t));
    for (int i = 0; i < count; ++i) p[i] = value;
    return p;
}

static relax_layer_dims tiny(void)
{
    relax_layer_dims d = {256, 4, 4, 64, 688, 32, 1e-5f, 10000.0f, 64, 2};
    return d;
}
static relax_layer_weights weights_of(const relax_layer_dims *d)
{
    const int hd = d->n_heads * d->head_dim, gd = d->n_kv_heads * d->head_dim;
    relax_layer_weights w;
    memset(&w, 0, sizeof w);
    w.wqkv = (relax_qmat){DEV, DEV, hd + 2 * gd, d->hidden, d->group};
    w.wo = (relax_qmat){DEV, DEV, d->hidden, hd, d->group};
    w.wgu = (relax_qmat){DEV, DEV, 2 * d->ffn, d->hidden, d->group};
    w.wdown = (relax_qmat){DEV, DEV, d->hidden, d->ffn, d->group};
    w.norm_attn = DEV, w.norm_ffn = DEV;
    return w;
}

int main(void)
{
    relax_layer_dims d = tiny();
    relax_layer_weights w = weights_of(&d);
    relax_kv_cache cache = {DEV, DEV, DEV};
    EXPECT_TRUE(relax_build_id() != NULL && strlen(relax_build_id()) > 0);

    /* ---- sizes: zero for anything invalid, monotone in the upper bounds ---- */
    EXPECT_TRUE(relax_workspace_bytes(NULL, 1, 1, 1) == 0);
    EXPECT_TRUE(relax_workspace_bytes(&d, 0, 64, 1) == 0);
    size_t prev = 0;
    const int rows[] = {1, 2, 15, 16, 17, 128, 129, 511, 2048};
    relax_layer_dims big = {4096, 32, 32, 128, 11008, 32, 1e-5f, 10000.0f, 4096, 64};
    relax_layer_dims gqa = {8192, 64, 8, 128, 28672, 32, 1e-5f, 10000.0f, 8192, 16};
    for (size_t i = 0; i < sizeof rows / sizeof rows[0]; ++i) {
        const size_t cur = relax_workspace_bytes(&big, rows[i], 4096, 1);
        EXPECT_TRUE(cur >= prev && cur > 0);
        prev = cur;
        EXPECT_TRUE(relax_workspace_bytes(&gqa, rows[i] > 64 ? 64 : rows[i], 8192, 16) > 0);
    }
    EXPECT_TRUE(relax_rope_table_bytes(&d) == (size_t)64 * 32 * 2 * 4);

    /* ---- the planner under both rules, entries at their exact count, one short, and absent ---- */
    const relax_layer_dims *shapes[] = {&d, &big, &gqa};
    for (int si = 0; si < 3; ++si)
        for (int rule = 0; rule <= 1; ++rule)
            for (size_t i = 0; i < sizeof rows / sizeof rows[0]; ++i) {
                const int n = rows[i] > shapes[si]->kv_capacity ? shapes[si]->kv_capacity : rows[i];
                int32_t count = 0;
                size_t planned = 0, unplanned = 0;
                EXPECT(relax_workspace_plan_rule(shapes[si], n, n, 1, rule, NULL, 0, &count, &planned, &unplanned), RELAX_OK);
                EXPECT_TRUE(count > 0 && planned > 0 && planned <= unplanned);
                relax_plan_entry *e = malloc((size_t)count * sizeof *e);
                int32_t count2 = 0;
                EXPECT(relax_workspace_plan_rule(shapes[si], n, n, 1, rule, e, count, &count2, &planned, &unplanned), RELAX_OK);
                EXPECT_TRUE(count2 == count);
                for (int t = 0; t < count; ++t) {
                    EXPECT_TRUE(memchr(e[t].name, 0, sizeof e[t].name) != NULL);
                    EXPECT_TRUE(e[t].bytes <= e[t].storage_bytes && e[t].offset % 256 == 0 && e[t].first_op <= e[t].last_op);
                }
                free(e);
                if (count > 1) {
                    e = malloc((size_t)(count - 1) * sizeof *e);
                    EXPECT(relax_workspace_plan_rule(shapes[si], n, n, 1, rule, e, count - 1, &count2, &planned, &unplanned), RELAX_ERR_WORKSPACE);
                    free(e);
                }
            }
    {
        int32_t count = 0;
        size_t a = 0, b = 0;
        EXPECT(relax_workspace_plan_rule(&d, 4, 4, 1, 2, NULL, 0, &count, &a, &b), RELAX_ERR_UNSUPPORTED);
        EXPECT(relax_workspace_plan(NULL, 4, 4, 1, NULL, 0, &count, &a, &b), RELAX_ERR_NULL);
        EXPECT(relax_workspace_plan(&d, 4, 4, 1, NULL, 0, NULL, &a, &b), RELAX_OK);          /* sizes only */
        EXPECT_TRUE(a > 0 && a <= b);
        EXPECT(relax_workspace_plan(&d, 0, 4, 1, NULL, 0, &count, &a, &b), RELAX_ERR_SHAPE);
    }

    /* ---- the layer call: every rejection happens before anything is enqueued ---- */
    const size_t wsb = relax_workspace_bytes(&d, 8, 64, 2);
    {
        int32_t *q3 = ints(1, 3), *l3 = ints(1, 3), *l2 = ints(1, 2), *l65 = ints(1, 65);
        relax_seqs ok = {1, q3, l3, NULL, NULL};
        EXPECT(relax_decoder_layer(NULL, &w, DEV, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_decoder_layer(&d, NULL, DEV, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_decoder_layer(&d, &w, NULL, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_decoder_layer(&d, &w, DEV, NULL, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, NULL, DEV, 3, DEV, wsb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &ok, NULL, 3, DEV, wsb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &ok, DEV, 3, NULL, wsb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &ok, DEV, 0, DEV, wsb, NULL), RELAX_ERR_SHAPE);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &ok, DEV, 4, DEV, wsb, NULL), RELAX_ERR_SHAPE);
        relax_seqs short_l = {1, q3, l2, NULL, NULL}, long_l = {1, q3, l65, NULL, NULL};
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &short_l, DEV, 3, DEV, wsb, NULL), RELAX_ERR_SHAPE);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &long_l, DEV, 3, DEV, wsb, NULL), RELAX_ERR_CAPACITY);
        int32_t *ones3 = ints(3, 1), *slot2 = ints(1, 2), *slotm = ints(1, -1);
        relax_seqs three = {3, ones3, ones3, NULL, NULL};                       /* two cache slots only */
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &three, DEV, 3, DEV, wsb, NULL), RELAX_ERR_CAPACITY);
        relax_seqs bad_slot = {1, q3, l3, slot2, NULL}, neg_slot = {1, q3, l3, slotm, NULL};
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &bad_slot, DEV, 3, DEV, wsb, NULL), RELAX_ERR_CAPACITY);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &neg_slot, DEV, 3, DEV, wsb, NULL), RELAX_ERR_CAPACITY);
        relax_seqs none = {0, q3, l3, NULL, NULL};
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &none, DEV, 3, DEV, wsb, NULL), RELAX_ERR_SHAPE);
        relax_layer_dims bad = d;
        bad.n_kv_heads = 3;
        EXPECT(relax_decoder_layer(&bad, &w, DEV, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_SHAPE);
        bad = d, bad.head_dim = 96;
        EXPECT(relax_decoder_layer(&bad, &w, DEV, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_UNSUPPORTED);
        bad = d, bad.group = 48;
        EXPECT(relax_decoder_layer(&bad, &w, DEV, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_UNSUPPORTED);
        bad = d, bad.group = 64;                                                /* matrices say 32 */
        EXPECT(relax_decoder_layer(&bad, &w, DEV, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_SHAPE);
        relax_layer_weights w2 = w;
        w2.wo.k = 128;
        EXPECT(relax_decoder_layer(&d, &w2, DEV, &cache, &ok, DEV, 3, DEV, wsb, NULL), RELAX_ERR_SHAPE);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &ok, DEV, 3, DEV, 0, NULL), RELAX_ERR_WORKSPACE);
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &ok, DEV, 3, (char *)DEV + 16, wsb, NULL), RELAX_ERR_WORKSPACE);
        int32_t *q8 = ints(1, 8), *l64 = ints(1, 64);
        relax_seqs full = {1, q8, l64, NULL, NULL};
        EXPECT(relax_decoder_layer(&d, &w, DEV, &cache, &full, DEV, 8, DEV, wsb - 1, NULL), RELAX_ERR_WORKSPACE);
        free(q3), free(l3), free(l2), free(l65), free(ones3), free(slot2), free(slotm), free(q8), free(l64);
    }

    /* ---- attention, with a workspace and with the library's static array ---- */
    {
        int32_t *q2 = ints(1, 2), *l5 = ints(1, 5), *l70 = ints(1, 70);
        relax_seqs s = {1, q2, l5, NULL, NULL}, over = {1, q2, l70, NULL, NULL};
        EXPECT(relax_attention(NULL, &cache, &s, &d, DEV, 2, DEV, 1 << 20, NULL), RELAX_ERR_NULL);
        EXPECT(relax_attention(DEV, &cache, &s, &d, DEV, 3, DEV, 1 << 20, NULL), RELAX_ERR_SHAPE);
        EXPECT(relax_attention(DEV, &cache, &over, &d, DEV, 2, DEV, 1 << 20, NULL), RELAX_ERR_CAPACITY);
        EXPECT(relax_attention(DEV, &cache, &s, &d, DEV, 2, DEV, 16, NULL), RELAX_ERR_WORKSPACE);
        EXPECT(relax_attention(DEV, &cache, &s, &d, DEV, 2, (char *)DEV + 128, 1 << 20, NULL), RELAX_ERR_WORKSPACE);
        EXPECT(relax_attention_static(NULL, &cache, &s, &d, DEV, 2, NULL), RELAX_ERR_NULL);
        EXPECT(relax_attention_static(DEV, &cache, &s, &d, DEV, 3, NULL), RELAX_ERR_SHAPE);
        EXPECT(relax_attention_static(DEV, &cache, &over, &d, DEV, 2, NULL), RELAX_ERR_CAPACITY);
        EXPECT_TRUE(relax_attention_static_max_bytes() == ((size_t)16 << 20));
        int32_t *q17 = ints(17, 1), *l17 = ints(17, 100);
        relax_layer_dims wide = gqa;
        wide.kv_slots = 64;
        relax_seqs many = {17, q17, l17, NULL, NULL};                           /* more than 16 sequences, no device table */
        EXPECT(relax_attention_static(DEV, &cache, &many, &wide, DEV, 17, NULL), RELAX_ERR_UNSUPPORTED);
        int32_t *q64 = ints(64, 1), *l64 = ints(64, 8192);
        relax_seqs huge = {64, q64, l64, NULL, DEV};                            /* partials beyond the static array */
        EXPECT(relax_attention_static(DEV, &cache, &huge, &wide, DEV, 64, NULL), RELAX_ERR_WORKSPACE);
        EXPECT(relax_rmsnorm_rope(NULL, NULL, NULL, 1, 256, 1e-5f, NULL, NULL, NULL, NULL, NULL), RELAX_ERR_NULL);
        EXPECT(relax_rmsnorm_rope(DEV, DEV, DEV, 0, 256, 1e-5f, NULL, NULL, NULL, NULL, NULL), RELAX_ERR_SHAPE);
        free(q2), free(l5), free(l70), free(q17), free(l17), free(q64), free(l64);
    }

    /* ---- matmul entry points and the decode exports ---- */
    {
        relax_qmat m = {DEV, DEV, 8, 64, 32};
        EXPECT(relax_dequant_matmul(NULL, &m, DEV, 1, NULL, 0, NULL), RELAX_ERR_NULL);
        EXPECT(relax_dequant_matmul(DEV, NULL, DEV, 1, NULL, 0, NULL), RELAX_ERR_NULL);
        EXPECT(relax_dequant_matmul(DEV, &m, DEV, 0, NULL, 0, NULL), RELAX_ERR_SHAPE);
        m.k = 60;
        EXPECT(relax_dequant_matmul(DEV, &m, DEV, 1, NULL, 0, NULL), RELAX_ERR_SHAPE);
        m.k = 64, m.group = 48;
        EXPECT(relax_dequant_matmul(DEV, &m, DEV, 1, NULL, 0, NULL), RELAX_ERR_UNSUPPORTED);
        EXPECT(relax_dequantize(&m, DEV, NULL), RELAX_ERR_UNSUPPORTED);
        m.group = 32, m.k = 12;
        EXPECT(relax_unpack_int4(&m, DEV, NULL), RELAX_ERR_SHAPE);
        relax_qmat tall = {DEV, DEV, 22016, 4096, 32};
        EXPECT_TRUE(relax_matmul_workspace_bytes(&tall, 128) == relax_matmul_workspace_bytes(&tall, 4096));
        EXPECT_TRUE(relax_matmul_workspace_bytes(NULL, 128) == 0);
        EXPECT(relax_half_matmul(NULL, DEV, DEV, 1, 8, 64, NULL), RELAX_ERR_NULL);
        EXPECT(relax_half_matmul(DEV, DEV, DEV, 1, 8, 60, NULL), RELAX_ERR_SHAPE);
        EXPECT(relax_half_matmul((const uint16_t *)((char *)DEV + 2), DEV, DEV, 1, 8, 64, NULL), RELAX_ERR_SHAPE);
        relax_qmat q3 = {DEV, DEV, 8, 60, 32};
        EXPECT(relax_unpack_q3(&q3, DEV, NULL), RELAX_ERR_SHAPE);                    /* k % 32 */
        EXPECT(relax_repack_q3(NULL, DEV, NULL), RELAX_ERR_NULL);
        EXPECT(relax_dequant_matmul_q3_native(DEV, NULL, DEV, 1, NULL), RELAX_ERR_NULL);
    }

    /* ---- the model step ---- */
    {
        relax_layer_weights layers[2] = {w, w};
        relax_model model = {d, 2, 100, layers, DEV, DEV, DEV};
        const size_t mb = relax_model_workspace_bytes(&model, 8, 64, 2);
        EXPECT_TRUE(mb > wsb);
        EXPECT_TRUE(relax_model_workspace_bytes(NULL, 8, 64, 2) == 0);
        relax_kv_cache caches[2] = {cache, cache};
        int32_t *q3 = ints(1, 3), *l3 = ints(1, 3), *l65 = ints(1, 65);
        relax_seqs s = {1, q3, l3, NULL, NULL}, over = {1, q3, l65, NULL, NULL};
        EXPECT(relax_model_step(NULL, DEV, caches, &s, DEV, DEV, 3, DEV, mb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_model_step(&model, NULL, caches, &s, DEV, DEV, 3, DEV, mb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_model_step(&model, DEV, NULL, &s, DEV, DEV, 3, DEV, mb, NULL), RELAX_ERR_NULL);
        EXPECT(relax_model_step(&model, DEV, caches, &s, DEV, DEV, 4, DEV, mb, NULL), RELAX_ERR_SHAPE);
        EXPECT(relax_model_step(&model, DEV, caches, &over, DEV, DEV, 3, DEV, mb, NULL), RELAX_ERR_CAPACITY);
        EXPECT(relax_model_step(&model, DEV, caches, &s, DEV, DEV, 3, DEV, 16, NULL), RELAX_ERR_WORKSPACE);
        EXPECT(relax_model_step(&model, DEV, caches, &s, DEV, DEV, 3, (char *)DEV + 64, mb, NULL), RELAX_ERR_WORKSPACE);
        relax_model bad = model;
        bad.vocab = 0;
        EXPECT(relax_model_step(&bad, DEV, caches, &s, DEV, DEV, 3, DEV, mb, NULL), RELAX_ERR_SHAPE);
        free(q3), free(l3), free(l65);
    }

    /* ---- options of the measurement header ---- */
    EXPECT(relax_set_option(NULL, 1), RELAX_ERR_NULL);
    EXPECT(relax_set_option("no_such_option", 1), RELAX_ERR_UNSUPPORTED);
    EXPECT(relax_set_option("gemm_waves_per_simd", 3), RELAX_ERR_SHAPE);
    EXPECT(relax_set_option("gemm_waves_per_simd", 2), RELAX_OK);
    EXPECT(relax_set_option("half_matmul_gemm_rows", -1), RELAX_ERR_SHAPE);

    if (failures) { fprintf(stderr, "%d expectation(s) failed\n", failures); return 1; }
    printf("abi driver ok\n");
    return 0;
}
