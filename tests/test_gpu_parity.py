"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI.

Bar: bit-exact for int4 decoding / indexing and for integer-valued contractions; within
|gpu - ref| <= 1e-2 + 2e-2 |ref| for fp16 results against the fp32 oracle."""
import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import assert_close, device_layer, f32_cache, oracle_dims, oracle_weights

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def rx():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2311_02103_amd import binding
    binding.lib()                      # raises if the HIP library is not built: no fallback exists
    return binding


def dev(a):
    from paper_2311_02103_amd.runtime import to_device
    return to_device(a)


def host_bits(t):
    from paper_2311_02103_amd.runtime import f16_bits
    return f16_bits(t)


def gpu_matmul(rx, x_bits, q, s, m, k, with_ws=False, group=32):
    """with_ws: bring the workspace that lets a few-row call take the split-K MFMA kernel."""
    n = x_bits.shape[0]
    out = torch.empty((n, m), dtype=torch.float16, device="cuda")
    qm = rx.QMat(dev(q), dev(s), m, k, group)
    ws, ws_bytes = None, 0
    if with_ws:
        ws_bytes = rx.relax_matmul_workspace_bytes(qm, n)
        ws = torch.full((max(ws_bytes, 16),), 0xFF, dtype=torch.uint8, device="cuda")       # NaN-pattern garbage
    rx.check(rx.relax_dequant_matmul(dev(x_bits), qm, out, n, ws, ws_bytes), "relax_dequant_matmul")
    torch.cuda.synchronize()
    return host_bits(out)


# ------------------------------------------------------------------------- decode exports: bit-exact
@pytest.mark.parametrize("m,k", [(5, 8), (33, 688), (64, 4096), (3, 11008)])
def test_unpack_and_dequantize_bit_exact(rx, m, k):
    r = np.random.RandomState(m * 7 + k)
    q = r.randint(0, 2 ** 32, size=(m, k // 8), dtype=np.uint64).astype(np.uint32)
    s = (r.randn(m, (k + 31) // 32) * 0.01).astype(np.float16).view(np.uint16)
    qm = rx.QMat(dev(q), dev(s), m, k)
    codes = torch.empty((m, k), dtype=torch.int8, device="cuda")
    dense = torch.empty((m, k), dtype=torch.float32, device="cuda")
    rx.check(rx.relax_unpack_int4(qm, codes), "relax_unpack_int4")
    rx.check(rx.relax_dequantize(qm, dense), "relax_dequantize")
    torch.cuda.synchronize()
    assert np.array_equal(codes.cpu().numpy(), oracle.unpack_int4(q, m, k))
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), oracle.dequantize(q, s, m, k).view(np.uint32))


# ------------------------------------------------------------------------- matvec: exact cases
@pytest.mark.parametrize("m,k,n", [(40, 256, 2), (65, 688, 3), (130, 4096, 1), (37, 11008, 2)])
def test_selector_matrix_bitwise(rx, m, k, n):
    # row r holds +1 (code 9) only at column (7r+3) mod k, scale 1  =>  out[i,r] = x[i,(7r+3) mod k].
    # x is integer-valued (every partial sum is exactly representable), so any (r,c) -> word / nibble /
    # scale-group indexing slip shows as a wrong integer; with N(0,1) x the result must still match to fp16 rounding.
    codes = np.full((m, k), 8, dtype=np.uint8)
    cols = (7 * np.arange(m) + 3) % k
    codes[np.arange(m), cols] = 9
    q = wl.pack_codes(codes)
    s = np.full((m, (k + 31) // 32), np.float16(1.0)).view(np.uint16)
    xi = ((np.arange(n)[:, None] * 5 + np.arange(k)[None, :] * 37) % 15 - 7).astype(np.float32)
    got = gpu_matmul(rx, xi.astype(np.float16).view(np.uint16), q, s, m, k).view(np.float16).astype(np.float32)
    assert np.array_equal(got, xi[:, cols])
    assert np.array_equal(got, oracle.dequant_matmul(xi, q, s, m, k))
    x = wl.normal_f16_bits(1, 77, (n, k))
    got = gpu_matmul(rx, x, q, s, m, k).view(np.float16).astype(np.float32)
    ref = oracle.dequant_matmul(wl.f16_bits_to_f32(x), q, s, m, k)
    assert np.array_equal(ref, wl.f16_bits_to_f32(x)[:, cols])
    assert np.abs(got - ref).max() <= 4e-3          # scale 1.0 here: ~150x the scale of real weights


@pytest.mark.parametrize("m,k,n", [(33, 688, 5), (64, 4096, 2), (31, 2048, 1), (16, 11008, 1),
                                   (70, 28672, 1), (19, 14336, 1)])       # rows split over the wavefronts of a workgroup
def test_integer_valued_matmul_bitwise(rx, m, k, n):
    r = np.random.RandomState(k + m)
    codes = r.randint(0, 16, size=(m, k)).astype(np.uint8)
    sc = r.choice([1.0, 2.0], size=(m, (k + 31) // 32)).astype(np.float16)
    # sparse small-integer x keeps |out| <= 2048 so the fp16 result is exact
    x = np.zeros((n, k), dtype=np.float32)
    hot = r.choice(k, size=24, replace=False)
    x[:, hot] = r.randint(-3, 4, size=(n, 24))
    xb = x.astype(np.float16).view(np.uint16)
    q, s = wl.pack_codes(codes), sc.view(np.uint16)
    ref = oracle.dequant_matmul(x, q, s, m, k)
    assert np.abs(ref).max() <= 2048
    got = gpu_matmul(rx, xb, q, s, m, k).view(np.float16).astype(np.float32)
    assert np.array_equal(got, ref)


# ------------------------------------------------------------------------- matvec: random data, tolerance
@pytest.mark.parametrize("m,k,n", [(768, 256, 37), (256, 256, 1), (1376, 256, 4), (256, 688, 37), (257, 688, 1),
                                   (1024, 4096, 1), (515, 4096, 17), (640, 11008, 1), (96, 11008, 3), (9, 8192, 2),
                                   (2, 28672, 1), (1, 64, 1),
                                   # rows that end in the first / second-to-last chunk of 2048 columns of the register-resident matvec
                                   (131, 2080, 1), (200, 4192, 1), (64, 8224, 1), (77, 2080, 3), (37, 10272, 1),
                                   # rows of 12289 .. 32768 columns (split over the four wavefronts of a workgroup): 14, 7, 10, 13 and
                                   # 6.75 chunks of 2048 columns, odd m, more pairs than workgroups, two rows of x
                                   (300, 5120, 1), (77, 6144, 3), (41, 4128, 2),      # three chunks of 2048 columns
                                   (300, 28672, 1), (131, 14336, 1), (64, 20480, 2), (37, 26624, 1), (1100, 13824, 1)])
def test_dequant_matmul_random(rx, m, k, n):
    q, s = wl.qmat(3, m * 131 + k, m, k)
    x = wl.normal_f16_bits(3, m + k + n, (n, k))
    ref = oracle.dequant_matmul(wl.f16_bits_to_f32(x), q, s, m, k)
    got = gpu_matmul(rx, x, q, s, m, k).view(np.float16).astype(np.float32)
    assert_close(got, ref, "dequant_matmul m=%d k=%d n=%d" % (m, k, n))
    # well inside the bar: fp32 accumulation, one fp16 rounding of the result
    assert np.abs(got - ref).max() <= 2e-3 * max(1.0, np.abs(ref).max())


def test_dequant_matmul_rows_are_independent(rx):
    m, k, n = 300, 4096, 5
    q, s = wl.qmat(4, 1, m, k)
    x = wl.normal_f16_bits(4, 2, (n, k))
    full = gpu_matmul(rx, x, q, s, m, k)
    for i in range(n):
        assert np.array_equal(gpu_matmul(rx, x[i:i + 1], q, s, m, k)[0], full[i])


# ------------------------------------------------------------------------- RMSNorm / rotary + append
def test_rmsnorm_and_rope_append(rx):
    shape = wl.TINY
    cap, n = 64, 6
    dims = rx.make_dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, cap, 2)
    od = oracle_dims(shape, cap)
    x = wl.normal_f16_bits(5, 1, (n, shape.hidden))
    w = wl.normal_f16_bits(5, 2, (shape.hidden,), std=0.1, mean=1.0)
    y = torch.empty((n, shape.hidden), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_rmsnorm_rope(dev(x), dev(w), y, n, shape.hidden, shape.rms_eps))
    torch.cuda.synchronize()
    assert_close(host_bits(y).view(np.float16), oracle.rmsnorm(wl.f16_bits_to_f32(x), w, shape.rms_eps), "rmsnorm")

    qkv = wl.normal_f16_bits(5, 3, (n, shape.qkv_rows))
    rope = torch.empty(rx.relax_rope_table_bytes(dims) // 4, dtype=torch.float32, device="cuda")
    rx.check(rx.relax_rope_table_init(dims, rope))
    kc = torch.full((2, cap, shape.n_kv_heads, shape.head_dim), float("nan"), dtype=torch.float16, device="cuda")
    vc = torch.full_like(kc, float("nan"))
    seqs_q, seqs_kv, slots = [2, 4], [40, 4], [1, 0]
    dq = dev(qkv)
    rx.check(rx.relax_rmsnorm_rope(None, None, None, n, shape.hidden, shape.rms_eps, qkv=dq, dims=dims,
                                   cache=rx.KVCache(kc, vc, rope), seqs=rx.Seqs(seqs_q, seqs_kv, slots)))
    torch.cuda.synchronize()
    Ko = np.full((2, cap, shape.n_kv_heads, shape.head_dim), np.nan, np.float32)
    Vo = Ko.copy()
    ref = oracle.rope_append(wl.f16_bits_to_f32(qkv), od, Ko, Vo, oracle.Seqs(seqs_q, seqs_kv, slots))
    assert_close(host_bits(dq).view(np.float16), ref, "rope qkv", atol=4e-3, rtol=2e-3)
    Kg, Vg = host_bits(kc).view(np.float16).astype(np.float32), host_bits(vc).view(np.float16).astype(np.float32)
    assert np.array_equal(np.isnan(Kg), np.isnan(Ko)) and np.array_equal(np.isnan(Vg), np.isnan(Vo))   # only the new rows
    mask = ~np.isnan(Ko)
    assert_close(Kg[mask], Ko[mask], "appended K", atol=4e-3, rtol=2e-3)
    assert np.array_equal(Vg[mask], Vo[mask])
    # the table itself: (cos, sin) of pos * base^(-2t/d) against float64
    tab = rope.cpu().numpy().reshape(cap, shape.head_dim // 2, 2)
    ang = np.arange(cap)[:, None] * shape.rope_base ** (-2.0 * np.arange(shape.head_dim // 2) / shape.head_dim)[None, :]
    assert np.abs(tab[:, :, 0] - np.cos(ang)).max() < 1e-7 and np.abs(tab[:, :, 1] - np.sin(ang)).max() < 1e-7


# ------------------------------------------------------------------------- attention
def run_attention(rx, h, g, d, cap, slots, q_lens, kv_lens, slot_ids, seed, poison=True):
    n = int(np.sum(q_lens))
    dims = rx.make_dims(h * d, h, g, d, 64, cap, slots)
    od = oracle.Dims(h * d, h, g, d, 64, kv_capacity=cap)
    kb, vb = (wl.normal_f16_bits(seed, 10 + j, (slots, cap, g, d)) for j in (0, 1))
    qb = wl.normal_f16_bits(seed, 12, (n, h, d))
    kc, vc = dev(kb).clone(), dev(vb).clone()
    if poison:      # nothing beyond each row's position may be read: poison the cache above every sequence's length
        for b, sl in enumerate(slot_ids):
            kc[sl, kv_lens[b]:] = float("nan")
            vc[sl, kv_lens[b]:] = float("nan")
    ws_bytes = rx.relax_workspace_bytes(dims, n, int(max(kv_lens)), len(q_lens))
    ws = torch.full((ws_bytes,), 0xFF, dtype=torch.uint8, device="cuda")       # NaN-pattern garbage in the scratch
    out = torch.empty((n, h, d), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_attention(dev(qb), rx.KVCache(kc, vc, None), rx.Seqs(q_lens, kv_lens, slot_ids), dims, out, n, ws,
                                ws_bytes), "relax_attention")
    torch.cuda.synchronize()
    ref = oracle.attention(wl.f16_bits_to_f32(qb), f32_cache(kb), f32_cache(vb), od, oracle.Seqs(q_lens, kv_lens, slot_ids))
    return host_bits(out).view(np.float16).astype(np.float32), ref


@pytest.mark.parametrize("L", [1, 2, 63, 64, 65, 257, 1000, 4096])
def test_decode_attention_lengths(rx, L):
    got, ref = run_attention(rx, 32, 32, 128, 4096, 1, [1], [L], [0], seed=20 + L)
    assert_close(got, ref, "decode attention L=%d" % L, atol=2e-3, rtol=1e-2)


@pytest.mark.parametrize("h,g,d", [(4, 4, 64), (8, 2, 64), (64, 8, 128), (6, 3, 128), (5, 5, 128), (12, 1, 64)])
def test_decode_attention_head_layouts(rx, h, g, d):
    got, ref = run_attention(rx, h, g, d, 600, 3, [1, 1, 1], [600, 1, 77], [2, 0, 1], seed=h * 10 + g)
    assert_close(got, ref, "attention h=%d g=%d d=%d" % (h, g, d), atol=2e-3, rtol=1e-2)


def test_attention_ragged_prefill_rows_and_many_sequences(rx):
    got, ref = run_attention(rx, 8, 4, 64, 128, 4, [5, 1, 37, 2], [9, 128, 37, 66], [3, 1, 0, 2], seed=31)
    assert_close(got, ref, "ragged attention", atol=2e-3, rtol=1e-2)
    B = 21                                         # more sequences than ride in kernel arguments: device table path
    kv = [int(v) for v in wl.uniform_lengths(32, B, 1, 300)]
    got, ref = run_attention(rx, 8, 8, 64, 300, B, [1] * B, kv, list(range(B))[::-1], seed=32)
    assert_close(got, ref, "21-sequence decode", atol=2e-3, rtol=1e-2)


@pytest.mark.parametrize("h,g,d,q_lens,kv_lens", [
    (4, 4, 128, [16], [16]),                      # smallest call that takes the MFMA kernel
    (4, 2, 128, [129], [129]),                    # one full q tile + one row; crosses a 64-token KV tile
    (2, 2, 64, [300], [300]),                     # head dim 64, several q tiles and KV tiles, ragged tails
    (4, 1, 128, [70], [333]),                     # chunked prefill: 263 cached tokens before the call's rows
    (8, 4, 64, [40, 1, 200, 17], [40, 90, 200, 64]),   # mixed batch: a decode row among prefills, different pasts
    (4, 4, 128, [150], [155]),                    # 5 cached tokens: the 32-token sub-tiles no longer line up with the 32-query groups, so
                                                  # a wavefront's second KV group meets sub-tiles that are masked entirely for its first queries
])
def test_prefill_attention_mfma(rx, h, g, d, q_lens, kv_lens):
    B = len(q_lens)
    got, ref = run_attention(rx, h, g, d, max(kv_lens) + 5, B, q_lens, kv_lens, list(range(B))[::-1], seed=40 + h + sum(q_lens))
    assert_close(got, ref, "prefill attention h=%d g=%d d=%d q=%s" % (h, g, d, q_lens), atol=2e-3, rtol=1e-2)


def test_prefill_attention_many_sequences_device_table(rx):
    B = 19                                        # more sequences than ride in kernel arguments
    q = [int(v) for v in wl.uniform_lengths(41, B, 1, 70)]
    q[3] = 33
    past = [int(v) for v in wl.uniform_lengths(42, B, 1, 50)]
    kv = [a + b - 1 for a, b in zip(q, past)]
    got, ref = run_attention(rx, 4, 2, 64, 128, B, q, kv, list(range(B)), seed=43)
    assert_close(got, ref, "19-sequence prefill", atol=2e-3, rtol=1e-2)


def test_prefill_attention_7b_2048_sampled_rows(rx):
    """Full cfg-3 shape (h=g=32, d=128, n=L=2048): the oracle computes sampled query rows one by one."""
    h = g = 32
    d, n, cap = 128, 2048, 2048
    dims = rx.make_dims(h * d, h, g, d, 64, cap, 1)
    od = oracle.Dims(h * d, h, g, d, 64, kv_capacity=cap)
    kb, vb = (wl.normal_f16_bits(50, 10 + j, (1, cap, g, d)) for j in (0, 1))
    qb = wl.normal_f16_bits(50, 12, (n, h, d))
    ws_bytes = rx.relax_workspace_bytes(dims, n, n, 1)
    ws = torch.full((ws_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    out = torch.empty((n, h, d), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_attention(dev(qb), rx.KVCache(dev(kb), dev(vb), None), rx.Seqs([n], [n], [0]), dims, out, n, ws, ws_bytes))
    torch.cuda.synchronize()
    got = host_bits(out).view(np.float16).astype(np.float32)
    assert np.isfinite(got).all()
    Kf, Vf = f32_cache(kb), f32_cache(vb)
    for row in (0, 1, 63, 64, 127, 128, 1000, 1983, 2047):
        # the same row as a decode call on the same cache: q_len 1, kv_len row+1
        ref = oracle.attention(wl.f16_bits_to_f32(qb[row:row + 1]), Kf, Vf, od, oracle.Seqs([1], [row + 1], [0]))
        assert_close(got[row:row + 1], ref, "prefill attention row %d" % row, atol=2e-3, rtol=1e-2)


# ------------------------------------------------------------------------- whole layer
def run_schedule(rx, shape, seed, cap, calls, slots=1, prefill_bits=None, n_max=None):
    """calls: list of (q_lens, kv_lens, slot_ids).  Returns per-call (gpu fp32, oracle fp32) and both caches."""
    w = wl.layer_weights(shape, seed)
    n_max = n_max or max(int(np.sum(c[0])) for c in calls)
    layer = device_layer(shape, w, cap, slots=slots, n_max=n_max, B_max=max(len(c[0]) for c in calls))
    od, ow = oracle_dims(shape, cap), oracle_weights(shape, w)
    cshape = (slots, cap, shape.n_kv_heads, shape.head_dim)
    if prefill_bits is not None:
        layer.load_cache(*prefill_bits)
        Ko, Vo = f32_cache(prefill_bits[0]).reshape(cshape), f32_cache(prefill_bits[1]).reshape(cshape)
    else:
        Ko, Vo = np.zeros(cshape, np.float32), np.zeros(cshape, np.float32)
    outs = []
    for ci, (ql, kl, sl) in enumerate(calls):
        n = int(np.sum(ql))
        x = wl.activations(shape, seed, ci, n)
        y = layer.forward(dev(x), ql, kl, sl)
        torch.cuda.synchronize()
        ref = oracle.decoder_layer(od, ow, x, Ko, Vo, oracle.Seqs(ql, kl, sl))
        outs.append((host_bits(y).view(np.float16).astype(np.float32), ref))
    Kg = host_bits(layer.k).view(np.float16).astype(np.float32)
    Vg = host_bits(layer.v).view(np.float16).astype(np.float32)
    return outs, (Kg, Vg), (Ko, Vo)


def test_tiny_layer_prefill_then_sixteen_decode_steps(rx):
    # workload 1: prefill n=37, then decode L=38..53, seed 0
    calls = [([37], [37], None)] + [([1], [L], None) for L in range(38, 54)]
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, wl.TINY, 0, 64, calls)
    for ci, (g, r) in enumerate(outs):
        assert_close(g, r, "tiny layer call %d" % ci)
    assert_close(Kg[:, :53], Ko[:, :53], "K cache", atol=5e-3, rtol=5e-3)
    assert_close(Vg[:, :53], Vo[:, :53], "V cache", atol=5e-3, rtol=5e-3)
    assert np.all(Kg[:, 53:] == 0) and np.all(Vg[:, 53:] == 0)               # nothing written beyond L


def test_tiny_layer_prefill_equals_sequential_decode_on_gpu(rx):
    shape, n = wl.TINY, 9
    w = wl.layer_weights(shape, 7)
    a = device_layer(shape, w, 16, n_max=n)
    b = device_layer(shape, w, 16, n_max=n)
    x = dev(wl.activations(shape, 7, 0, n))
    full = a.forward(x, [n], [n])
    steps = torch.cat([b.forward(x[i:i + 1], [1], [i + 1]) for i in range(n)])
    torch.cuda.synchronize()
    assert_close(host_bits(steps).view(np.float16), host_bits(full).view(np.float16).astype(np.float32), "prefill vs decode")


def test_tiny_layer_ragged_batch(rx):
    calls = [([3, 5, 1], [3, 5, 1], [2, 0, 1]), ([1, 1, 1], [4, 6, 2], [2, 0, 1]), ([2, 1], [8, 3], [0, 1])]
    outs, _, _ = run_schedule(rx, wl.TINY, 3, 32, calls, slots=3)
    for ci, (g, r) in enumerate(outs):
        assert_close(g, r, "ragged call %d" % ci)


def test_layer_zero_projections_return_input(rx):
    # zero Wo and Wdown: both residual branches vanish and the layer is the identity.  The fast matvec removes the
    # decode offset per group in fp32 (sum x (1024+u) - 1032 sum x), so a zero matrix gives ~1e-6, not a bitwise 0.
    shape = wl.TINY
    w = wl.layer_weights(shape, 9)
    w["wo.q"] = np.full_like(w["wo.q"], 0x88888888)
    w["wdown.q"] = np.full_like(w["wdown.q"], 0x88888888)
    layer = device_layer(shape, w, 8, n_max=4)
    x = wl.activations(shape, 9, 0, 4)
    y = layer.forward(dev(x), [4], [4])
    torch.cuda.synchronize()
    assert_close(host_bits(y).view(np.float16), wl.f16_bits_to_f32(x), "identity layer", atol=1e-4, rtol=1e-3)


@pytest.mark.parametrize("L", [1, 300, 449, 2231, 4096])      # 449: first length with 8 splits; 2231: ragged last step of every split
def test_llama7b_layer_decode(rx, L):
    shape, cap = wl.LLAMA7B, 4096
    pre = wl.kv_prefill(shape, 1, 1, cap)
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, shape, 1, cap, [([1], [L], None)], prefill_bits=pre)
    g, r = outs[0]
    assert_close(g, r, "7B decode layer L=%d" % L)
    assert_close(Kg[0, L - 1], Ko[0, L - 1], "appended K", atol=5e-3, rtol=5e-3)
    assert_close(Vg[0, L - 1], Vo[0, L - 1], "appended V", atol=5e-3, rtol=5e-3)


def test_llama7b_layer_prefill_17(rx):
    outs, _, _ = run_schedule(rx, wl.LLAMA7B, 2, 64, [([17], [17], None)])
    assert_close(*outs[0], "7B prefill n=17")


# ------------------------------------------------------------------------- one decode row over a pre-filled cache, more shapes
FAST_SMALL = wl.LayerShape("small-fast", hidden=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn=704)
FAST_MID = wl.LayerShape("mid-fast", hidden=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn=5632)
# hidden width of the 13B shape (5120 = 2.5 chunks of 2048 columns: the three-chunk variants, attention merge folded in), small FFN
H5120 = wl.LayerShape("h5120", hidden=5120, n_heads=40, n_kv_heads=40, head_dim=128, ffn=1024)


@pytest.mark.parametrize("shape,cap,Ls", [(FAST_SMALL, 600, [1, 2, 63, 64, 65, 130, 600]),
                                          (FAST_MID, 2100, [1, 777, 2100]),
                                          (H5120, 700, [1, 64, 449, 700]),
                                          (wl.LLAMA7B, 4096, [2, 2048, 4095])])
def test_one_decode_row_over_a_prefilled_cache(rx, shape, cap, Ls):
    pre = wl.kv_prefill(shape, 11, 1, cap)
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, shape, 11, cap, [([1], [L], None) for L in Ls], prefill_bits=pre)
    for ci, (g, r) in enumerate(outs):
        assert_close(g, r, "%s decode L=%d" % (shape.name, Ls[ci]))
    for L in Ls:                                                    # appended K/V rows
        assert_close(Kg[0, L - 1], Ko[0, L - 1], "K row %d" % (L - 1), atol=5e-3, rtol=5e-3)
        assert_close(Vg[0, L - 1], Vo[0, L - 1], "V row %d" % (L - 1), atol=5e-3, rtol=5e-3)


def test_repeated_decode_call_is_reproducible_and_raises_no_flag(rx):
    shape, cap = FAST_MID, 512
    w = wl.layer_weights(shape, 5)
    layer = device_layer(shape, w, cap)
    layer.load_cache(*wl.kv_prefill(shape, 5, 1, cap))
    x = dev(wl.activations(shape, 5, 0, 1))
    ys = [host_bits(layer.forward(x, [1], [300])).copy() for _ in range(5)]         # same call five times: same bits
    torch.cuda.synchronize()
    for y in ys[1:]:
        assert np.array_equal(y, ys[0])
    assert rx.relax_workspace_error(layer.dims, layer.ws) == 0


# ------------------------------------------------------------------------- MFMA GEMM path (n >= 16, k % 128 == 0)
@pytest.mark.parametrize("m,k,n", [(64, 128, 16), (260, 256, 33), (512, 4096, 128), (256, 11008, 17), (1024, 1024, 511),
                                   # two launches: the first 8192 weight rows on 256 x 256 tiles (one full round of them at 2048
                                   # rows of x), the last 256 on 128 x 256 tiles
                                   (8448, 256, 2048)])
def test_gemm_integer_valued_bitwise(rx, m, k, n):
    r = np.random.RandomState(m + k + n)
    codes = r.randint(0, 16, size=(m, k)).astype(np.uint8)
    sc = r.choice([1.0, 2.0], size=(m, k // 32)).astype(np.float16)
    x = np.zeros((n, k), dtype=np.float32)
    for i in range(n):                                   # sparse small-integer rows keep |out| <= 2048: exact in fp16
        hot = r.choice(k, size=20, replace=False)
        x[i, hot] = r.randint(-3, 4, size=20)
    q, s = wl.pack_codes(codes), sc.view(np.uint16)
    ref = oracle.dequant_matmul(x, q, s, m, k)
    assert np.abs(ref).max() <= 2048
    got = gpu_matmul(rx, x.astype(np.float16).view(np.uint16), q, s, m, k).view(np.float16).astype(np.float32)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("m,k,n", [(768, 256, 37), (4096, 4096, 16), (1024, 4096, 129), (512, 11008, 64), (12288, 4096, 40)])
def test_gemm_random_against_oracle_and_matvec_path(rx, m, k, n):
    q, s = wl.qmat(6, m * 7 + k, m, k)
    x = wl.normal_f16_bits(6, n, (n, k))
    ref = oracle.dequant_matmul(wl.f16_bits_to_f32(x), q, s, m, k)
    got = gpu_matmul(rx, x, q, s, m, k).view(np.float16).astype(np.float32)
    assert_close(got, ref, "gemm m=%d k=%d n=%d" % (m, k, n))
    assert np.abs(got - ref).max() <= 3e-3 * max(1.0, np.abs(ref).max())
    # the same rows through the matrix-vector kernel (n below the dispatch threshold): both paths meet the same bar
    rows = gpu_matmul(rx, x[:3], q, s, m, k).view(np.float16).astype(np.float32)
    assert_close(rows, ref[:3], "matvec rows")


# ------------------------------------------------------------------------- few-row split-K MFMA kernel (2 <= n <= 64, k % 256 == 0)
@pytest.mark.parametrize("m,k,n", [(128, 256, 2), (100, 512, 5), (260, 1024, 16), (512, 4096, 32), (132, 11008, 33), (1024, 2048, 64),
                                   (260, 512, 65), (512, 4096, 128), (132, 11008, 100),
                                   # above 128 rows with a workspace: the tiled GEMM, cut along k where its tiles are few
                                   (516, 4096, 129), (1000, 11008, 300), (260, 2048, 512)])
def test_skinny_integer_valued_bitwise(rx, m, k, n):
    r = np.random.RandomState(m + k + n)
    codes = r.randint(0, 16, size=(m, k)).astype(np.uint8)
    sc = r.choice([1.0, 2.0], size=(m, k // 32)).astype(np.float16)
    x = np.zeros((n, k), dtype=np.float32)
    for i in range(n):                                   # sparse small-integer rows keep |out| <= 2048: exact in fp16
        hot = r.choice(k, size=20, replace=False)
        x[i, hot] = r.randint(-3, 4, size=20)
    q, s = wl.pack_codes(codes), sc.view(np.uint16)
    ref = oracle.dequant_matmul(x, q, s, m, k)
    assert np.abs(ref).max() <= 2048
    got = gpu_matmul(rx, x.astype(np.float16).view(np.uint16), q, s, m, k, with_ws=True).view(np.float16).astype(np.float32)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("m,k,n", [(768, 256, 3), (4096, 4096, 16), (8192, 8192, 16), (512, 28672, 7), (12288, 4096, 40), (1000, 1024, 64),
                                   (4096, 4096, 128), (1000, 11008, 97), (768, 256, 65),
                                   (4096, 4096, 200), (4096, 11008, 130), (8192, 1024, 511)])     # k-split tiled GEMM (8, 8 and 2 splits)
def test_skinny_random_against_oracle_and_reproducible(rx, m, k, n):
    q, s = wl.qmat(8, m * 7 + k, m, k)
    x = wl.normal_f16_bits(8, n, (n, k))
    ref = oracle.dequant_matmul(wl.f16_bits_to_f32(x), q, s, m, k)
    got = gpu_matmul(rx, x, q, s, m, k, with_ws=True)
    assert_close(got.view(np.float16).astype(np.float32), ref, "skinny m=%d k=%d n=%d" % (m, k, n))
    assert np.abs(got.view(np.float16).astype(np.float32) - ref).max() <= 3e-3 * max(1.0, np.abs(ref).max())
    # partial tiles are summed in a fixed order: a second run gives the same bits
    assert np.array_equal(got, gpu_matmul(rx, x, q, s, m, k, with_ws=True))


def test_mid_layer_batched_decode_through_the_few_row_kernel(rx):
    """Ragged batches of 2..16 decode rows (and a 40-row mixed call) on the mid-size layer: the matrix path with the
    split-K kernel, norm / rope / attention as separate launches."""
    B = 16
    past = [int(v) for v in wl.uniform_lengths(33, B, 1, 90)]
    kb, vb = wl.kv_prefill(FAST_MID, 33, B, 128)
    calls = [([1] * B, [p + 1 for p in past], list(range(B))),
             ([1, 1], [past[3] + 2, past[7] + 2], [3, 7]),
             ([1] * 5, [past[b] + (3 if b in (3, 7) else 2) for b in (0, 3, 5, 7, 9)], [0, 3, 5, 7, 9]),
             ([20, 1, 19], [past[1] + 21, past[2] + 2, past[4] + 20], [1, 2, 4])]
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, FAST_MID, 33, 128, calls, slots=B, prefill_bits=(kb, vb))
    for i, (got, ref) in enumerate(outs):
        assert_close(got, ref, "batched call %d" % i)


def test_mid_layer_prefill_and_decode_through_gemm_and_matvec(rx):
    calls = [([37], [37], None), ([1], [38], None), ([16], [54], None), ([130], [184], None)]
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, FAST_MID, 21, 256, calls)
    for ci, (g, r) in enumerate(outs):
        assert_close(g, r, "mid layer call %d" % ci)
    assert_close(Kg[:, :184], Ko[:, :184], "K cache", atol=5e-3, rtol=5e-3)
    assert_close(Vg[:, :184], Vo[:, :184], "V cache", atol=5e-3, rtol=5e-3)


def test_wide_layer_decode_rows_through_the_long_row_matvec(rx):
    """A layer whose attention width (112 heads x 128 = 14336) and FFN width (13824) exceed what one wavefront keeps of x: at
    one row the output projection (fp32 residual epilogue) and the down projection (fp16 residual epilogue) run the matvec
    that splits a row over the wavefronts of a workgroup; the attention merge is a launch of its own at that width."""
    shape = wl.LayerShape("wide", hidden=512, n_heads=112, n_kv_heads=112, head_dim=128, ffn=13824)
    calls = [([5], [5], None), ([1], [6], None), ([1], [7], None)]
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, shape, 29, 16, calls)
    for ci, (g, r) in enumerate(outs):
        assert_close(g, r, "wide layer call %d" % ci)
    assert_close(Kg[:, :7], Ko[:, :7], "K cache", atol=5e-3, rtol=5e-3)
    assert_close(Vg[:, :7], Vo[:, :7], "V cache", atol=5e-3, rtol=5e-3)


def test_llama7b_layer_prefill_128(rx):
    outs, _, _ = run_schedule(rx, wl.LLAMA7B, 2, 128, [([128], [128], None)])
    assert_close(*outs[0], "7B prefill n=128")


def test_13b_width_layer_two_to_four_decode_rows_on_the_matvec_kernels(rx):
    """Hidden 5120 and FFN 13824 (the 13B widths, fewer heads' worth of rows would not change the kernels): two to four decode
    rows through the three-chunk matvec variants (two rows of x per pass) and the long-row kernel (two and four rows per pass)."""
    shape = wl.LayerShape("w13b", hidden=5120, n_heads=40, n_kv_heads=40, head_dim=128, ffn=13824)
    past = [int(v) for v in wl.uniform_lengths(43, 4, 1, 40)]
    kb, vb = wl.kv_prefill(shape, 43, 4, 48)
    calls = [([1, 1], [past[0] + 1, past[1] + 1], [0, 1]),
             ([1, 1, 1], [past[2] + 1, past[0] + 2, past[3] + 1], [2, 0, 3]),
             ([1, 1, 1, 1], [past[1] + 2, past[3] + 2, past[2] + 2, past[0] + 3], [1, 3, 2, 0])]
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, shape, 43, 48, calls, slots=4, prefill_bits=(kb, vb))
    for ci, (g, r) in enumerate(outs):
        assert_close(g, r, "13B-width layer, %d decode rows" % (ci + 2))
    assert_close(Kg, Ko, "K cache", atol=5e-3, rtol=5e-3)
    assert_close(Vg, Vo, "V cache", atol=5e-3, rtol=5e-3)


@pytest.mark.parametrize("matvec_rows", [1, 4])
def test_llama7b_layer_two_to_five_decode_rows_on_both_paths(rx, matvec_rows):
    """Batches of two to five decode rows of the 7B-shaped layer through the matvec kernels with several rows per pass
    (the default up to four rows) and, with the switch at 1, through the few-row matrix path: both against the oracle."""
    rx.check(rx.relax_set_option("layer_matvec_rows", matvec_rows))
    try:
        past = [int(v) for v in wl.uniform_lengths(41, 5, 1, 60)]
        kb, vb = wl.kv_prefill(wl.LLAMA7B, 41, 5, 64)
        calls = [([1, 1], [past[0] + 1, past[1] + 1], [0, 1]),
                 ([1, 1, 1], [past[2] + 1, past[0] + 2, past[4] + 1], [2, 0, 4]),
                 ([1, 1, 1, 1], [past[1] + 2, past[3] + 1, past[2] + 2, past[4] + 2], [1, 3, 2, 4]),
                 ([1] * 5, [past[0] + 3, past[1] + 3, past[2] + 3, past[3] + 2, past[4] + 3], [0, 1, 2, 3, 4])]
        outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, wl.LLAMA7B, 41, 64, calls, slots=5, prefill_bits=(kb, vb))
        for ci, (g, r) in enumerate(outs):
            assert_close(g, r, "7B layer, %d decode rows, layer_matvec_rows = %d" % (ci + 2, matvec_rows))
        assert_close(Kg, Ko, "K cache", atol=5e-3, rtol=5e-3)
        assert_close(Vg, Vo, "V cache", atol=5e-3, rtol=5e-3)
    finally:
        rx.check(rx.relax_set_option("layer_matvec_rows", 4))


def test_llama7b_layer_row_counts_around_the_dispatch_boundaries(rx):
    """The same binary picks the kernels from n: up to four rows of a small model stay on the matvec kernels (two or
    four rows of x share one pass over the weights), five take the few-row path; at 64 rows every matmul is the few-row
    kernel, at 65 and 96 the tall gate/up matrix goes to the tiled GEMM while the other three stay (their finishing
    passes still fold the light steps)."""
    calls = [([40, 25], [40, 25], [0, 1]),            # 65 rows, two prefills
             ([1, 1], [41, 26], [0, 1]),              # two decode rows
             ([1, 1, 1], [42, 27, 1], [0, 1, 2]),     # three
             ([64], [64], [3]), ([96], [96], [2])]
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, wl.LLAMA7B, 5, 100, calls, slots=4, n_max=96)
    for ci, (g, r) in enumerate(outs):
        assert_close(g, r, "7B dispatch boundaries, call %d" % ci)
    assert_close(Kg, Ko, "K cache", atol=5e-3, rtol=5e-3)
    assert_close(Vg, Vo, "V cache", atol=5e-3, rtol=5e-3)


@pytest.mark.parametrize("n", [200, 511, 2048])
def test_llama7b_layer_prefill_full_sizes(rx, n):
    """The remaining row counts of the symbolic-n configuration, every row and the whole appended cache against the
    oracle (200: the tiled GEMM of the output and down projections is cut along k into 4 splits, finished by the few-row
    kernel's finishing pass; 511: ragged tiles everywhere, 2 splits; 2048: the size the prefill figures are quoted on)."""
    outs, (Kg, Vg), (Ko, Vo) = run_schedule(rx, wl.LLAMA7B, 2, n, [([n], [n], None)])
    assert_close(*outs[0], "7B prefill n=%d" % n)
    assert_close(Kg[0, :n], Ko[0, :n], "appended K", atol=5e-3, rtol=5e-3)
    assert_close(Vg[0, :n], Vo[0, :n], "appended V", atol=5e-3, rtol=5e-3)


# ------------------------------------------------------------------------- fp16-weight matmul (matvec passes / tiled GEMM without decode)
def gpu_half_matmul(rx, x_bits, w_bits):
    n, k = x_bits.shape
    m = w_bits.shape[0]
    out = torch.empty((n, m), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_half_matmul(dev(x_bits), dev(w_bits), out, n, m, k), "relax_half_matmul")
    torch.cuda.synchronize()
    return host_bits(out).view(np.float16).astype(np.float32)


@pytest.mark.parametrize("m,k,n", [(512, 1024, 1), (1000, 4096, 3), (516, 4096, 8), (516, 4096, 9), (1000, 4096, 11), (1000, 4096, 12),
                                   (4096, 4096, 17), (300, 1024, 64), (260, 2048, 65), (1028, 11008, 130), (4096, 4096, 300),
                                   (700, 1024, 513), (250, 1000, 40), (1000, 4096 + 64, 40)])      # the last two: shapes the GEMM cannot take
def test_half_matmul_against_oracle(rx, m, k, n):
    """Plain fp16 weights through the same dispatch on n: passes of up to 8 rows through the matvec kernel below the
    crossover, the tiled MFMA GEMM without its decode step from there on (every tile shape, ragged edges), and the
    matvec passes again for matrices the GEMM cannot take (m % 4 != 0, k % 128 != 0)."""
    w = wl.normal_f16_bits(9, m * 3 + k, (m, k))
    w = (wl.f16_bits_to_f32(w) * 0.02).astype(np.float16).view(np.uint16)          # weight scale of the int4 workloads
    x = wl.normal_f16_bits(9, n + k, (n, k))
    ref = oracle.half_matmul(wl.f16_bits_to_f32(x), w)
    got = gpu_half_matmul(rx, x, w)
    assert_close(got, ref, "half_matmul m=%d k=%d n=%d" % (m, k, n))
    assert np.abs(got - ref).max() <= 2e-3 * max(1.0, np.abs(ref).max())


def test_half_matmul_both_kernels_on_the_same_rows(rx):
    """The crossover is a tuning value: forcing the GEMM down to one row, or the matvec passes up to 40 rows, changes the
    kernel, not the result beyond the fp16 bar."""
    m, k, n = 2048, 4096, 40
    w = (wl.f16_bits_to_f32(wl.normal_f16_bits(10, 1, (m, k))) * 0.02).astype(np.float16).view(np.uint16)
    x = wl.normal_f16_bits(10, 2, (n, k))
    ref = oracle.half_matmul(wl.f16_bits_to_f32(x), w)
    try:
        for rows in (1, 10 ** 6):
            rx.check(rx.relax_set_option("half_matmul_gemm_rows", rows))
            for nn in (1, 5, 40):
                assert_close(gpu_half_matmul(rx, x[:nn], w), ref[:nn], "half_matmul, GEMM from %d rows, n=%d" % (rows, nn))
    finally:
        rx.check(rx.relax_set_option("half_matmul_gemm_rows", 0))         # back to the default: by estimate
