"""Host-side contract of the C ABI: the library loads without a GPU, exports every declared symbol,
and every shape / pointer check fires before anything is enqueued (Relax Sec. 3.2 / 4.1: shape
constraints are checked at the function boundary and raise errors)."""
import os
import re

import pytest

from paper_2311_02103_amd import binding as rx

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = 0x10000   # a non-null fake device address: every call below must fail validation before touching it


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))) if h.endswith(".h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)       # declarations only: comments also name calls
    declared = set(re.findall(r"\b(relax_[a-z0-9_]+)\s*\(", header))
    declared -= {"relax_status", "relax_stream"}
    assert declared == set(rx.EXPORTS), declared ^ set(rx.EXPORTS)
    lib = rx.lib()
    for name in declared:
        assert getattr(lib, name) is not None
    assert "gfx950" in rx.relax_build_id()


def dims(**kw):
    base = dict(hidden=256, n_heads=4, n_kv_heads=4, head_dim=64, ffn=688, kv_capacity=64, kv_slots=2)
    base.update(kw)
    return rx.make_dims(**base)


def weights(d, **kw):
    H, F = d.hidden, d.ffn
    hd, qkvw = d.n_heads * d.head_dim, (d.n_heads + 2 * d.n_kv_heads) * d.head_dim
    m = dict(wqkv=rx.QMat(P, P, qkvw, H), wo=rx.QMat(P, P, H, hd), wgu=rx.QMat(P, P, 2 * F, H), wdown=rx.QMat(P, P, H, F))
    m.update(kw)
    return rx.LayerWeights(m["wqkv"], m["wo"], m["wgu"], m["wdown"], P, P)


def test_workspace_query():
    d = dims()
    small, big = rx.relax_workspace_bytes(d, 1, 64, 1), rx.relax_workspace_bytes(d, 37, 64, 2)
    assert 0 < small < big
    assert rx.relax_workspace_bytes(None, 1, 1, 1) == 0
    assert rx.relax_workspace_bytes(dims(head_dim=96), 1, 1, 1) == 0
    assert rx.relax_workspace_bytes(d, 0, 64, 1) == 0
    assert rx.relax_rope_table_bytes(d) == 64 * 32 * 2 * 4
    # monotone in every symbolic upper bound
    prev = 0
    for n in (1, 2, 17, 128, 2048):
        cur = rx.relax_workspace_bytes(dims(hidden=4096, n_heads=32, n_kv_heads=32, head_dim=128, ffn=11008,
                                            kv_capacity=4096), n, 4096, 1)
        assert cur >= prev
        prev = cur


def test_dequant_matmul_checks():
    assert rx.relax_dequant_matmul(None, rx.QMat(P, P, 8, 64), P, 1) == rx.ERR_NULL
    assert rx.relax_dequant_matmul(P, None, P, 1) == rx.ERR_NULL
    assert rx.relax_dequant_matmul(P, rx.QMat(None, P, 8, 64), P, 1) == rx.ERR_NULL
    assert rx.relax_dequant_matmul(P, rx.QMat(P, P, 8, 64), None, 1) == rx.ERR_NULL
    assert rx.relax_dequant_matmul(P, rx.QMat(P, P, 8, 64), P, 0) == rx.ERR_SHAPE
    assert rx.relax_dequant_matmul(P, rx.QMat(P, P, 8, 60), P, 1) == rx.ERR_SHAPE       # k % 8
    assert rx.relax_dequant_matmul(P, rx.QMat(P, P, 0, 64), P, 1) == rx.ERR_SHAPE
    assert rx.relax_dequant_matmul(P, rx.QMat(P, P, 8, 1 << 20), P, 1) == rx.ERR_UNSUPPORTED


def test_decoder_layer_checks():
    d = dims()
    w = weights(d)
    ws_bytes = rx.relax_workspace_bytes(d, 8, 64, 2)
    call = lambda dd, ww, sq, n, x=P, ws=P, wsb=ws_bytes, cache=rx.KVCache(P, P, P): \
        rx.relax_decoder_layer(dd, ww, x, cache, sq, P, n, ws, wsb)
    ok_seq = rx.Seqs([3], [3])
    assert call(None, w, ok_seq, 3) == rx.ERR_NULL
    assert call(d, None, ok_seq, 3) == rx.ERR_NULL
    assert call(d, w, None, 3) == rx.ERR_NULL
    assert call(d, w, ok_seq, 3, x=None) == rx.ERR_NULL
    assert call(d, w, ok_seq, 3, cache=rx.KVCache(P, P, None)) == rx.ERR_NULL
    assert call(d, w, ok_seq, 3, ws=None) == rx.ERR_NULL
    assert call(d, w, ok_seq, 0) == rx.ERR_SHAPE
    assert call(d, w, ok_seq, 4) == rx.ERR_SHAPE                          # sum q_lens != n
    assert call(d, w, rx.Seqs([3], [2]), 3) == rx.ERR_SHAPE              # L < q_len
    assert call(d, w, rx.Seqs([3, 0], [3, 0]), 3) == rx.ERR_SHAPE        # empty sequence
    assert call(d, w, rx.Seqs([3], [65]), 3) == rx.ERR_CAPACITY          # L > capacity
    assert call(d, w, rx.Seqs([1, 1, 1], [1, 1, 1]), 3) == rx.ERR_CAPACITY   # third slot does not exist
    assert call(d, w, rx.Seqs([3], [3], slots=[2]), 3) == rx.ERR_CAPACITY
    assert call(d, w, rx.Seqs([3], [3], slots=[-1]), 3) == rx.ERR_CAPACITY
    assert call(dims(n_kv_heads=3), w, ok_seq, 3) == rx.ERR_SHAPE        # h % g
    assert call(dims(head_dim=96), w, ok_seq, 3) == rx.ERR_UNSUPPORTED
    assert call(dims(group=64), w, ok_seq, 3) == rx.ERR_SHAPE             # matrices of group 32 in a layer of group 64
    assert call(dims(group=48), w, ok_seq, 3) == rx.ERR_UNSUPPORTED
    assert call(d, weights(d, wo=rx.QMat(P, P, 256, 128)), ok_seq, 3) == rx.ERR_SHAPE    # matrix does not fit dims
    assert call(d, weights(d, wdown=rx.QMat(P, P, 256, 684)), ok_seq, 3) == rx.ERR_SHAPE  # k % 8
    assert call(d, w, rx.Seqs([8], [64]), 8, wsb=ws_bytes - 1) == rx.ERR_WORKSPACE
    assert call(d, w, rx.Seqs([8], [64]), 8, wsb=0) == rx.ERR_WORKSPACE


def test_attention_and_norm_rope_checks():
    d = dims()
    c = rx.KVCache(P, P, P)
    s = rx.Seqs([2], [5])
    assert rx.relax_attention(None, c, s, d, P, 2, P, 1 << 20) == rx.ERR_NULL
    assert rx.relax_attention(P, c, None, d, P, 2, P, 1 << 20) == rx.ERR_NULL
    assert rx.relax_attention(P, c, s, d, P, 3, P, 1 << 20) == rx.ERR_SHAPE
    assert rx.relax_attention(P, c, rx.Seqs([2], [70]), d, P, 2, P, 1 << 20) == rx.ERR_CAPACITY
    assert rx.relax_attention(P, c, s, d, P, 2, P, 16) == rx.ERR_WORKSPACE
    assert rx.relax_rmsnorm_rope(None, None, None, 1, 256, 1e-5) == rx.ERR_NULL
    assert rx.relax_rmsnorm_rope(P, None, P, 1, 256, 1e-5) == rx.ERR_NULL
    assert rx.relax_rmsnorm_rope(P, P, P, 0, 256, 1e-5) == rx.ERR_SHAPE
    assert rx.relax_rmsnorm_rope(None, None, None, 2, 256, 1e-5, qkv=P, dims=d, cache=rx.KVCache(P, P, None), seqs=s) == rx.ERR_NULL
    assert rx.relax_rmsnorm_rope(None, None, None, 2, 256, 1e-5, qkv=P, dims=d, cache=c, seqs=rx.Seqs([1], [5])) == rx.ERR_SHAPE
    assert rx.relax_unpack_int4(rx.QMat(P, P, 4, 12), P) == rx.ERR_SHAPE
    assert rx.relax_dequantize(rx.QMat(P, None, 4, 16), P) == rx.ERR_NULL
    assert rx.relax_rope_table_init(d, None) == rx.ERR_NULL


def test_workspace_pointers_must_be_256_byte_aligned():
    d = dims()
    w = weights(d)
    c = rx.KVCache(P, P, P)
    s = rx.Seqs([2], [5])
    big = 1 << 24
    assert rx.relax_decoder_layer(d, w, P, c, s, P, 2, P + 16, big) == rx.ERR_WORKSPACE
    assert rx.relax_attention(P, c, s, d, P, 2, P + 128, big) == rx.ERR_WORKSPACE
    assert rx.relax_workspace_init(d, P + 8, big) == rx.ERR_WORKSPACE
    m = rx.Model(d, [w], 100, P, P, P)
    assert rx.relax_model_step(m, P, [c], s, P, P, 2, P + 64, big) == rx.ERR_WORKSPACE


def test_static_attention_checks():
    """The entry point without a workspace refuses, on the host, what its fixed device array cannot hold."""
    d = dims()
    c = rx.KVCache(P, P, P)
    s = rx.Seqs([2], [5])
    assert rx.relax_attention_static_max_bytes() == 16 << 20
    assert rx.relax_attention_static(None, c, s, d, P, 2) == rx.ERR_NULL
    assert rx.relax_attention_static(P, c, None, d, P, 2) == rx.ERR_NULL
    assert rx.relax_attention_static(P, c, s, d, P, 3) == rx.ERR_SHAPE
    assert rx.relax_attention_static(P, c, rx.Seqs([2], [70]), d, P, 2) == rx.ERR_CAPACITY
    big = dims(hidden=8192, n_heads=64, n_kv_heads=8, head_dim=128, ffn=28672, kv_capacity=8192, kv_slots=64)
    # 17 sequences without a device table: the copy of the descriptor would need a workspace
    assert rx.relax_attention_static(P, c, rx.Seqs([1] * 17, [100] * 17), big, P, 17) == rx.ERR_UNSUPPORTED
    # 64 rows x 64 heads x 16 splits x 130 floats = 34 MB of partials: beyond the 16 MiB array
    assert rx.relax_attention_static(P, c, rx.Seqs([1] * 64, [8192] * 64, device_table=P), big, P, 64) == rx.ERR_WORKSPACE


def test_model_step_and_matmul_workspace_checks():
    d = dims()
    w = weights(d)
    model = lambda **kw: rx.Model(kw.get("d", d), kw.get("layers", [w, w]), kw.get("vocab", 100), kw.get("emb", P), kw.get("norm", P),
                                  kw.get("head", P))
    m = model()
    wsb = rx.relax_model_workspace_bytes(m, 8, 64, 2)
    assert wsb > rx.relax_workspace_bytes(d, 8, 64, 2)                    # the layer workspace plus activations and logits
    assert rx.relax_model_workspace_bytes(None, 8, 64, 2) == 0
    assert rx.relax_model_workspace_bytes(model(vocab=0), 8, 64, 2) == 0
    assert rx.relax_model_workspace_bytes(m, 0, 64, 2) == 0
    caches = [rx.KVCache(P, P, P)] * 2
    seq = rx.Seqs([3], [3])
    call = lambda mm=m, ids=P, cc=caches, sq=seq, n=3, ws=P, b=wsb: rx.relax_model_step(mm, ids, cc, sq, P, P, n, ws, b)
    assert call(mm=None) == rx.ERR_NULL
    assert call(ids=None) == rx.ERR_NULL
    assert call(cc=None) == rx.ERR_NULL
    assert call(ws=None) == rx.ERR_NULL
    assert call(mm=model(emb=None)) == rx.ERR_NULL
    assert call(mm=model(head=None)) == rx.ERR_NULL
    assert call(cc=[rx.KVCache(P, P, P), rx.KVCache(P, None, P)]) == rx.ERR_NULL
    assert call(mm=model(vocab=0)) == rx.ERR_SHAPE
    assert call(mm=model(d=dims(hidden=252))) == rx.ERR_SHAPE            # hidden % 8
    assert call(mm=model(layers=[w, weights(d, wo=rx.QMat(P, P, 256, 128))])) == rx.ERR_SHAPE
    assert call(n=4) == rx.ERR_SHAPE                                      # sum q_lens != n
    assert call(sq=rx.Seqs([3], [65])) == rx.ERR_CAPACITY
    assert call(b=rx.relax_model_workspace_bytes(m, 3, 3, 1) - 1) == rx.ERR_WORKSPACE     # one byte short of what this very call needs
    assert call(b=16) == rx.ERR_WORKSPACE
    # a model without layers needs no caches
    assert rx.relax_model_step(model(layers=[]), None, None, seq, P, P, 3, P, wsb) == rx.ERR_NULL        # ids still required
    # few-row matmul workspace: zero for bad arguments, grows with the row bound up to the kernel's limit
    q = rx.QMat(P, P, 4096, 4096)
    assert rx.relax_matmul_workspace_bytes(None, 4) == 0 and rx.relax_matmul_workspace_bytes(q, 0) == 0
    assert 0 < rx.relax_matmul_workspace_bytes(q, 2) < rx.relax_matmul_workspace_bytes(q, 64)
    assert rx.relax_matmul_workspace_bytes(q, 128) == rx.relax_matmul_workspace_bytes(q, 4096)
    assert rx.relax_matmul_workspace_bytes(rx.QMat(P, P, 64, 688), 16) == 0      # k not a multiple of 256: the kernel never runs
    # probes validate before launching
    assert rx.relax_probe_stream_read(None, 64, P) == rx.ERR_NULL
    assert rx.relax_probe_stream_read(P + 4, 64, P) == rx.ERR_SHAPE
    assert rx.relax_probe_mfma(None, 10, False)[0] == rx.ERR_NULL


def test_half_matmul_checks():
    assert rx.relax_half_matmul(None, P, P, 1, 8, 64) == rx.ERR_NULL
    assert rx.relax_half_matmul(P, None, P, 1, 8, 64) == rx.ERR_NULL
    assert rx.relax_half_matmul(P, P, None, 1, 8, 64) == rx.ERR_NULL
    assert rx.relax_half_matmul(P, P, P, 0, 8, 64) == rx.ERR_SHAPE
    assert rx.relax_half_matmul(P, P, P, 1, 0, 64) == rx.ERR_SHAPE
    assert rx.relax_half_matmul(P, P, P, 1, 8, 60) == rx.ERR_SHAPE          # k % 8
    assert rx.relax_half_matmul(P + 2, P, P, 1, 8, 64) == rx.ERR_SHAPE      # x not 16-byte aligned
    assert rx.relax_half_matmul(P, P, P, 1, 8, 80000) == rx.ERR_UNSUPPORTED  # a row of x beyond the matvec kernel's LDS
    assert rx.relax_set_option("half_matmul_gemm_rows", -1) == rx.ERR_SHAPE


def test_dispatch_options_check_their_ranges():
    for name, bad, good in (("layer_matvec_rows", (0, 65), 4), ("layer_matvec_mb", (-1, 4097), 96)):
        for v in bad:
            assert rx.relax_set_option(name, v) == rx.ERR_SHAPE
        assert rx.relax_set_option(name, good) == rx.OK
    assert rx.relax_set_option("no_such_option", 1) == rx.ERR_UNSUPPORTED


def test_no_product_module_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2311_02103_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_unsupported_group_is_refused():
    assert rx.relax_dequant_matmul(P, rx.QMat(P, P, 8, 64, 48), P, 1) == rx.ERR_UNSUPPORTED
    assert rx.relax_dequantize(rx.QMat(P, P, 8, 64, 16), P) == rx.ERR_UNSUPPORTED
    assert rx.relax_workspace_bytes(rx.make_dims(256, 4, 4, 64, 688, 64, 1, group=96), 1, 1, 1) == 0


def test_layer_rejects_a_matrix_whose_group_differs_from_the_dims():
    d = rx.make_dims(256, 4, 4, 64, 688, 64, 2, group=64)
    good = lambda m, k: rx.QMat(P, P, m, k, 64)
    w = rx.LayerWeights(good(768, 256), good(256, 256), rx.QMat(P, P, 1376, 256, 32), good(256, 688), P, P)
    assert rx.relax_decoder_layer(d, w, P, rx.KVCache(P, P, P), rx.Seqs([1], [1]), P, 1, P, 1 << 24) == rx.ERR_SHAPE
