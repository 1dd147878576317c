"""Pins for the CPU oracle: every check compares it with something other than itself --
hand-packed words (tests/golden), closed forms, invariants, library routines in
float64 and brute force on tiny shapes.  No GPU, no HIP library involved.

The paper (Relax, arXiv 2311.02103) prints no numeric example for this path
(its decode_q4 case study, Sec. 4.2 / Fig. 9, is a figure); the pins therefore
come from the format's definition and from mathematics.
"""
import os

import numpy as np
import pytest
import scipy.special

import oracle
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")
RS = np.random.RandomState


def f16(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def ones_scales(m, k, value=1.0):
    return np.full((m, (k + 31) // 32), np.float16(value)).view(np.uint16)


# ----------------------------------------------------------------------------- fp16 decode
def test_half_to_float_all_patterns_match_ieee_library():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


# ----------------------------------------------------------------------------- unpack / indexing
def _golden_words():
    rows = []
    for line in open(os.path.join(GOLD, "int4_words.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        word, vals = line.split(":")
        rows.append((int(word, 16), [int(v) for v in vals.split()]))
    assert len(rows) >= 12
    return rows


def test_unpack_hand_packed_words():
    for word, vals in _golden_words():
        got = oracle.unpack_int4(np.array([[word]], dtype=np.uint32), 1, 8)
        assert got.tolist() == [vals], hex(word)


def test_unpack_word_and_row_addressing():
    # all codes 8 (zero) except one nibble: element (r, c) must be the only non-zero
    m, k = 5, 48
    for (r, c) in [(0, 0), (0, 7), (0, 8), (2, 31), (3, 32), (4, 47), (1, 19)]:
        q = np.full((m, k // 8), 0x88888888, dtype=np.uint32)
        q[r, c // 8] = (0x88888888 & ~(0xF << (4 * (c % 8)))) | (0xD << (4 * (c % 8)))
        got = oracle.unpack_int4(q, m, k)
        want = np.zeros((m, k), dtype=np.int8)
        want[r, c] = 5
        assert np.array_equal(got, want), (r, c)


@pytest.mark.parametrize("m,k", [(40, 256), (64, 688), (9, 24)])
def test_selector_matrix_picks_columns_bitwise(m, k):
    # row r holds +1 (code 9) only at column (7r+3) mod k, scale 1  =>  out[i,r] = x[i,(7r+3) mod k]
    codes = np.full((m, k), 8, dtype=np.uint8)
    cols = (7 * np.arange(m) + 3) % k
    codes[np.arange(m), cols] = 9
    q = wl.pack_codes(codes)
    x = RS(1).randn(3, k).astype(np.float32)
    out = oracle.dequant_matmul(x, q, ones_scales(m, k), m, k)
    assert np.array_equal(out.view(np.uint32), x[:, cols].view(np.uint32))


def test_pack_codes_generator_against_hand_packed_words():
    for word, vals in _golden_words():
        codes = (np.array([vals], dtype=np.int16) + 8).astype(np.uint8)
        assert int(wl.pack_codes(codes)[0, 0]) == word


# ----------------------------------------------------------------------------- dequant
@pytest.mark.parametrize("k", [64, 688])
def test_dequant_group_scales_are_powers_of_two(k):
    m = 3
    G = (k + 31) // 32
    codes = np.full((m, k), 10, dtype=np.uint8)            # +2 everywhere
    expo = (np.arange(m)[:, None] * 3 + np.arange(G)[None, :]) % 24 - 12
    scales = np.ldexp(np.float32(1), expo).astype(np.float16).view(np.uint16)
    W = oracle.dequantize(wl.pack_codes(codes), scales, m, k)
    want = 2.0 * np.ldexp(1.0, expo)[:, np.arange(k) // 32]
    assert np.array_equal(W, want.astype(np.float32))


def test_dequant_is_exact_product_for_all_codes_and_odd_scales():
    m, k = 4, 64
    codes = (np.arange(m * k).reshape(m, k) % 16).astype(np.uint8)
    sc = np.array([[0.3331, 1.7], [0.004513, 3.0e-5], [65504.0, 6.0e-8], [1.0, 0.0]], dtype=np.float32)
    sb = f16(sc)
    W = oracle.dequantize(wl.pack_codes(codes), sb, m, k)
    want = (codes.astype(np.float64) - 8) * sb.view(np.float16).astype(np.float64)[:, np.arange(k) // 32]
    assert np.array_equal(W.astype(np.float64), want)      # 4-bit x 11-bit product is exact in fp32


# ----------------------------------------------------------------------------- other quantisation groups (64, 128 columns per scale)
def _golden_group_cases():
    cases = []
    for line in open(os.path.join(GOLD, "group_scales.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        head, rest = line.split(":")
        per_row, pairs = rest.split("|")
        group, k = (int(v) for v in head.split())
        cases.append((group, k, int(per_row), [tuple(int(v) for v in pr.split("->")) for pr in pairs.split()]))
    assert len(cases) >= 6
    return cases


def test_group_scale_indexing_against_hand_worked_table():
    """Scale number g of a row holds 2^(g - 8) and every code is +1: the decoded element IS its scale, so the element at
    column c names the scale it read.  Columns and expected scale numbers come from the hand-written table."""
    for group, k, per_row, pairs in _golden_group_cases():
        m = 3
        assert (k + group - 1) // group == per_row
        expo = np.arange(per_row)[None, :] - 8 + np.arange(m)[:, None] * 0          # same powers in every row ...
        scales = np.ldexp(np.float32(1), expo).astype(np.float16)
        scales[1] *= np.float16(4.0)                                                 # ... except row 1: rows must not mix
        W = oracle.dequantize(wl.pack_codes(np.full((m, k), 9, np.uint8)), scales.view(np.uint16), m, k, group)
        for c, g in pairs:
            assert W[0, c] == 2.0 ** (g - 8) and W[2, c] == 2.0 ** (g - 8), (group, k, c, g)
            assert W[1, c] == 4.0 * 2.0 ** (g - 8), (group, k, c, g)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("k", [256, 688])
def test_wider_group_equals_group_32_with_repeated_scales(group, k):
    """A matrix with one scale per `group` columns is the group-32 matrix whose neighbouring scales are equal: decode and
    matmul through the wider-group entry points must equal, bit for bit, the (separately pinned) group-32 ones on scales
    repeated group/32 times -- including the short last group of k = 688."""
    m, n = 9, 3
    q, s = wl.qmat(21, group, m, k, group=group)
    assert s.shape == (m, (k + group - 1) // group)
    s32 = np.repeat(s, group // 32, axis=1)[:, :(k + 31) // 32].copy()
    assert np.array_equal(oracle.dequantize(q, s, m, k, group).view(np.uint32), oracle.dequantize(q, s32, m, k).view(np.uint32))
    x = RS(22).randn(n, k).astype(np.float32)
    assert np.array_equal(oracle.dequant_matmul(x, q, s, m, k, group).view(np.uint32), oracle.dequant_matmul(x, q, s32, m, k).view(np.uint32))


@pytest.mark.parametrize("group", [64, 128])
def test_wider_group_matmul_integer_case_and_float64(group):
    m, k, n = 17, 688, 4
    r = RS(23 + group)
    codes = r.randint(0, 16, size=(m, k)).astype(np.uint8)
    sc = r.choice([1.0, 2.0], size=(m, (k + group - 1) // group)).astype(np.float32)
    x = r.randint(-3, 4, size=(n, k)).astype(np.float32)
    out = oracle.dequant_matmul(x, wl.pack_codes(codes), f16(sc), m, k, group)
    W = (codes.astype(np.int64) - 8) * np.repeat(sc.astype(np.int64), group, axis=1)[:, :k]
    assert np.array_equal(out.astype(np.int64), x.astype(np.int64) @ W.T)
    q, s = wl.qmat(24, group, m, k, group=group)
    xr = r.randn(n, k).astype(np.float32)
    dense = (oracle.unpack_int4(q, m, k).astype(np.float64) * np.repeat(s.view(np.float16).astype(np.float64), group, axis=1)[:, :k])
    want = xr.astype(np.float64) @ dense.T
    got = oracle.dequant_matmul(xr, q, s, m, k, group)
    assert np.max(np.abs(got - want)) < 2e-5 * max(1.0, np.max(np.abs(want)))


@pytest.mark.parametrize("group", [64, 128])
def test_quantizer_with_wider_groups(group):
    m, k = 6, 688
    w = wl.normal_f32(25, group, (m, k), std=0.02)
    q, s = wl.quantize_q4(w, group)
    G = (k + group - 1) // group
    assert s.shape == (m, G)
    W = oracle.dequantize(q, s, m, k, group)
    sc = np.repeat(s.view(np.float16).astype(np.float32), group, axis=1)[:, :k]
    assert np.all(np.abs(w - W) <= 0.5 * sc * (1 + 2e-3) + 1e-12)
    codes = np.abs(oracle.unpack_int4(q, m, k).astype(np.int32))
    for g in range(G):
        assert np.all(codes[:, g * group:min(k, (g + 1) * group)].max(axis=1) == 7)
    amax = np.abs(np.pad(w, ((0, 0), (0, G * group - k))).reshape(m, G, group)).max(axis=2)
    assert np.array_equal(s, (amax / np.float32(7.0)).astype(np.float16).view(np.uint16))


def test_layer_with_group_64_equals_layer_with_repeated_group_32_scales():
    shape, cap, group = wl.TINY, 16, 64
    w = wl.layer_weights(shape, 26, group=group)
    mats = shape.matrices()
    wide = oracle.LayerWeights(*(oracle.QMat(w[n + ".q"], w[n + ".s"], *mats[n], group) for n in ("wqkv", "wo", "wgu", "wdown")),
                               w["norm_attn"], w["norm_ffn"])
    rep = lambda nme: np.repeat(w[nme + ".s"], 2, axis=1)[:, :(mats[nme][1] + 31) // 32].copy()
    narrow = oracle.LayerWeights(*(oracle.QMat(w[n + ".q"], rep(n), *mats[n]) for n in ("wqkv", "wo", "wgu", "wdown")),
                                 w["norm_attn"], w["norm_ffn"])
    dims = oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.rms_eps, shape.rope_base, cap)
    x = wl.activations(shape, 26, 0, 5)
    outs = []
    for lw in (wide, narrow):
        K, V = np.zeros((1, cap, shape.n_kv_heads, shape.head_dim), np.float32), np.zeros((1, cap, shape.n_kv_heads, shape.head_dim), np.float32)
        outs.append(oracle.decoder_layer(dims, lw, x, K, V, oracle.Seqs([5], [5])))
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32)) and np.abs(outs[0]).max() > 0.1


# ----------------------------------------------------------------------------- matmul
def test_matmul_all_ones_closed_form():
    m, k, n = 6, 688, 2
    for u, s in [(9, 1.0), (15, 0.5), (0, 2.0), (3, 0.25)]:
        q = wl.pack_codes(np.full((m, k), u, dtype=np.uint8))
        out = oracle.dequant_matmul(np.ones((n, k), np.float32), q, ones_scales(m, k, s), m, k)
        assert np.all(out == k * (u - 8) * s)


def test_matmul_integer_case_is_exact():
    m, k, n = 33, 688, 5
    r = RS(2)
    codes = r.randint(0, 16, size=(m, k)).astype(np.uint8)
    sc = r.choice([1.0, 2.0], size=(m, (k + 31) // 32)).astype(np.float32)
    x = r.randint(-3, 4, size=(n, k)).astype(np.float32)
    out = oracle.dequant_matmul(x, wl.pack_codes(codes), f16(sc), m, k)
    W = (codes.astype(np.int64) - 8) * sc.astype(np.int64)[:, np.arange(k) // 32]
    want = x.astype(np.int64) @ W.T
    assert np.array_equal(out.astype(np.int64), want) and np.all(out == np.round(out))


@pytest.mark.parametrize("m,k,n", [(17, 256, 4), (8, 688, 3)])
def test_matmul_against_float64_library_gemm(m, k, n):
    q, s = wl.qmat(5, 1, m, k)
    x = RS(3).randn(n, k).astype(np.float32)
    W = oracle.dequantize(q, s, m, k).astype(np.float64)   # pinned above
    want = x.astype(np.float64) @ W.T
    got = oracle.dequant_matmul(x, q, s, m, k)
    assert np.max(np.abs(got - want)) <= 2e-6 * np.sqrt(k) * np.max(np.abs(want)) + 1e-7
    # transposed-operand / swapped-index mistakes: out must be [n, m]
    assert got.shape == (n, m)


def test_half_matmul_against_float64():
    r = RS(4)
    w = f16(r.randn(11, 40) * 0.02)
    x = r.randn(3, 40).astype(np.float32)
    want = x.astype(np.float64) @ w.view(np.float16).astype(np.float64).T
    assert np.allclose(oracle.half_matmul(x, w), want, rtol=1e-5, atol=1e-6)


# ----------------------------------------------------------------------------- quantiser (input generator)
@pytest.mark.parametrize("m,k", [(16, 256), (7, 688)])
def test_quantizer_error_bound_range_and_idempotence(m, k):
    w = wl.normal_f32(11, 9, (m, k), std=0.02)
    w[2, 32:64] = 0.0                                      # an all-zero group
    q, s = wl.quantize_q4(w)
    assert q.shape == (m, k // 8) and s.shape == (m, (k + 31) // 32)
    codes = oracle.unpack_int4(q, m, k).astype(np.int32)
    W = oracle.dequantize(q, s, m, k)
    sc = s.view(np.float16).astype(np.float32)[:, np.arange(k) // 32]
    assert np.all(np.abs(w - W) <= 0.5 * sc * (1 + 2e-3) + 1e-12)
    assert codes.min() >= -7 and codes.max() <= 7
    G = (k + 31) // 32
    for r in range(m):
        for g in range(G):
            blk = np.abs(codes[r, g * 32:min(k, (g + 1) * 32)])
            if (r, g) == (2, 1):
                assert blk.max() == 0 and s.view(np.float16)[r, g] == 0
            else:
                assert blk.max() == 7
    q2, s2 = wl.quantize_q4(W)
    assert np.array_equal(s2, s) and np.array_equal(q2, q)


# ----------------------------------------------------------------------------- RMSNorm
def test_rmsnorm_constant_row_closed_form():
    H, eps = 96, 1e-5
    w = f16(1 + 0.1 * RS(5).randn(H))
    wf = w.view(np.float16).astype(np.float64)
    for c in (0.5, -3.0, 1e-3):
        y = oracle.rmsnorm(np.full((2, H), c, np.float32), w, eps)
        want = c / np.sqrt(c * c + eps) * wf
        assert np.allclose(y, want[None, :], rtol=3e-6, atol=0)


def test_rmsnorm_scale_invariance_unit_weight_rms_and_float64():
    H, eps = 256, 1e-5
    r = RS(6)
    x = r.randn(3, H).astype(np.float32)
    one = f16(np.ones(H))
    y = oracle.rmsnorm(x, one, eps)
    ms = (x.astype(np.float64) ** 2).mean(axis=1)
    assert np.allclose(np.sqrt((y.astype(np.float64) ** 2).mean(axis=1)), np.sqrt(ms / (ms + eps)), rtol=1e-6)
    assert np.allclose(oracle.rmsnorm(64 * x, one, eps), y, rtol=2e-5, atol=1e-6)
    w = f16(1 + 0.1 * r.randn(H))
    want = x / np.sqrt(ms + eps)[:, None] * w.view(np.float16).astype(np.float64)
    assert np.allclose(oracle.rmsnorm(x, w, eps), want, rtol=3e-6, atol=1e-7)
    # eps sits inside the square root: a zero row maps to zero, not NaN
    assert np.all(oracle.rmsnorm(np.zeros((1, H), np.float32), w, eps) == 0)


# ----------------------------------------------------------------------------- RoPE
def test_rope_identity_norm_unit_vector_and_relative_property():
    d, base = 64, 10000.0
    r = RS(7)
    v = r.randn(d).astype(np.float32)
    assert np.array_equal(oracle.rope(v, 0, base).view(np.uint32), v.view(np.uint32))
    for pos in (1, 37, 4095, 8000):
        o = oracle.rope(v, pos, base).astype(np.float64)
        h = d // 2
        assert np.allclose(o[:h] ** 2 + o[h:] ** 2, v[:h].astype(np.float64) ** 2 + v[h:].astype(np.float64) ** 2,
                           rtol=1e-5)
        for t in (0, 1, 5, h - 1):                      # partner of t is t + d/2, frequency base^(-2t/d)
            e = np.zeros(d, np.float32)
            e[t] = 1.0
            o = oracle.rope(e, pos, base)
            ang = pos * base ** (-2.0 * t / d)
            want = np.zeros(d)
            want[t], want[t + h] = np.cos(ang), np.sin(ang)
            assert np.allclose(o, want, atol=2e-7), (pos, t)
            e = np.zeros(d, np.float32)
            e[t + h] = 1.0
            o = oracle.rope(e, pos, base)
            want = np.zeros(d)
            want[t], want[t + h] = -np.sin(ang), np.cos(ang)
            assert np.allclose(o, want, atol=2e-7), (pos, t)
    q, k = r.randn(d).astype(np.float32), r.randn(d).astype(np.float32)
    ref = float(oracle.rope(q, 9, base).astype(np.float64) @ oracle.rope(k, 4, base).astype(np.float64))
    for shift in (1, 100, 3000):
        val = float(oracle.rope(q, 9 + shift, base).astype(np.float64)
                    @ oracle.rope(k, 4 + shift, base).astype(np.float64))
        assert abs(val - ref) < 1e-4 * (1 + abs(ref))


# ----------------------------------------------------------------------------- attention
def _cache(r, slots, cap, g, d):
    return (r.randn(slots, cap, g, d).astype(np.float32), r.randn(slots, cap, g, d).astype(np.float32))


def _attn_f64(q, K, V, dims, seqs):
    """float64 reference with library softmax; one (row, head) at a time."""
    n = q.shape[0]
    h, g, d = dims.n_heads, dims.n_kv_heads, dims.head_dim
    out = np.zeros((n, h, d))
    row = 0
    for b in range(len(seqs.q)):
        slot = b if seqs.sl is None else int(seqs.sl[b])
        for i in range(int(seqs.q[b])):
            pos = int(seqs.kv[b]) - int(seqs.q[b]) + i
            for j in range(h):
                kv = j // (h // g)
                Kt = K[slot, :pos + 1, kv, :].astype(np.float64)
                Vt = V[slot, :pos + 1, kv, :].astype(np.float64)
                p = scipy.special.softmax(Kt @ q[row, j].astype(np.float64) / np.sqrt(d))
                out[row, j] = p @ Vt
            row += 1
    return out


def test_attention_softmax_rows_sum_to_one_and_float64():
    r = RS(8)
    dims = oracle.Dims(256, 4, 2, 16, 64, kv_capacity=40)
    K, V = _cache(r, 3, 40, 2, 16)
    seqs = oracle.Seqs([5, 1, 3], [9, 40, 3], slots=[2, 0, 1])
    q = r.randn(9, 4, 16).astype(np.float32)
    out, probs = oracle.attention(q, K, V, dims, seqs, want_probs=True)
    want = _attn_f64(q, K, V, dims, seqs)
    assert np.allclose(out, want, rtol=1e-5, atol=1e-6)
    row = 0
    for b in range(3):
        for i in range(int(seqs.q[b])):
            pos = int(seqs.kv[b]) - int(seqs.q[b]) + i
            p = probs[row, :, :pos + 1]
            assert np.allclose(p.sum(axis=1), 1.0, atol=1e-6) and np.all(p >= 0)
            assert np.all(np.isnan(probs[row, :, pos + 1:]))      # never written beyond pos
            row += 1


def test_attention_special_cases():
    r = RS(9)
    dims = oracle.Dims(64, 2, 2, 8, 16, kv_capacity=12)
    K, V = _cache(r, 1, 12, 2, 8)
    q = r.randn(1, 2, 8).astype(np.float32)
    # L = 1: output is V[0] exactly
    out = oracle.attention(q, K, V, dims, oracle.Seqs([1], [1]))
    assert np.array_equal(out[0], V[0, 0])
    # q = 0: uniform weights -> mean of V over t <= pos
    out = oracle.attention(np.zeros_like(q), K, V, dims, oracle.Seqs([1], [7]))
    assert np.allclose(out[0], V[0, :7].mean(axis=0), rtol=1e-6, atol=1e-7)
    # one overwhelming score -> that V row
    K2 = K.copy()
    K2[0, 4, 1, :] = 200.0 * q[0, 1] / np.linalg.norm(q[0, 1])
    out = oracle.attention(q, K2, V, dims, oracle.Seqs([1], [9]))
    assert np.allclose(out[0, 1], V[0, 4, 1], atol=1e-5)
    # scale is 1/sqrt(d): with K rows = c * q / |q|^2 * sqrt(d) the scores are exactly c
    c = np.array([0.0, 1.0, 2.0], dtype=np.float64)
    K3 = K.copy()
    for t in range(3):
        K3[0, t, 0, :] = (c[t] * q[0, 0] / (q[0, 0].astype(np.float64) @ q[0, 0]) * np.sqrt(8)).astype(np.float32)
    out = oracle.attention(q, K3, V, dims, oracle.Seqs([1], [3]))
    p = np.exp(c) / np.exp(c).sum()
    assert np.allclose(out[0, 0], p @ V[0, :3, 0].astype(np.float64), rtol=1e-5, atol=1e-6)


def test_attention_causal_mask_nan_poison_invariance():
    r = RS(10)
    dims = oracle.Dims(64, 4, 4, 8, 16, kv_capacity=16)
    K, V = _cache(r, 2, 16, 4, 8)
    seqs = oracle.Seqs([4, 1], [6, 10])
    q = r.randn(5, 4, 8).astype(np.float32)
    base = oracle.attention(q, K, V, dims, seqs)
    Kp, Vp = K.copy(), V.copy()
    Kp[0, 6:], Vp[0, 6:], Kp[1, 10:], Vp[1, 10:] = np.nan, np.nan, np.nan, np.nan
    assert np.array_equal(oracle.attention(q, Kp, Vp, dims, seqs), base)
    # row 0 of sequence 0 sits at pos 2: entries 3.. (later rows of the same call) must not matter
    Kp[0, 3:], Vp[0, 3:] = np.nan, np.nan
    got = oracle.attention(q, Kp, Vp, dims, seqs)
    assert np.array_equal(got[0], base[0]) and np.isnan(got[1]).all()


def test_attention_gqa_equals_mha_on_replicated_heads():
    r = RS(11)
    h, g, d, cap = 8, 2, 8, 10
    K, V = _cache(r, 1, cap, g, d)
    q = r.randn(3, h, d).astype(np.float32)
    seqs = oracle.Seqs([3], [10])
    a = oracle.attention(q, K, V, oracle.Dims(64, h, g, d, 16, kv_capacity=cap), seqs)
    Kr, Vr = np.repeat(K, h // g, axis=2), np.repeat(V, h // g, axis=2)
    b = oracle.attention(q, np.ascontiguousarray(Kr), np.ascontiguousarray(Vr),
                         oracle.Dims(64, h, h, d, 16, kv_capacity=cap), seqs)
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------- SwiGLU
def test_swiglu_identities():
    z = np.array([[0.0, 1.5, -1.5, 30.0, -30.0, 0.25]], dtype=np.float32)
    up = np.array([[3.0, 1.0, 1.0, 2.0, 1.0, -4.0]], dtype=np.float32)
    a = oracle.swiglu(np.concatenate([z, up], axis=1))[0].astype(np.float64)
    assert a[0] == 0.0
    assert abs((a[1] - a[2]) - 1.5) < 1e-6                 # silu(z) - silu(-z) = z
    assert abs(a[3] - 60.0) < 1e-5 and abs(a[4]) < 1e-10   # silu(z) -> z, silu(-z) -> 0
    want = z[0].astype(np.float64) * scipy.special.expit(z[0].astype(np.float64)) * up[0]
    assert np.allclose(a, want, rtol=1e-6, atol=1e-12)
    # layout is [gate (F) ; up (F)], not interleaved
    gu = np.array([[1.0, 2.0, 10.0, 100.0]], dtype=np.float32)
    a = oracle.swiglu(gu)[0]
    assert np.allclose(a, [1 / (1 + np.exp(-1)) * 10, 2 / (1 + np.exp(-2)) * 100], rtol=1e-6)


# ----------------------------------------------------------------------------- whole layer
def _tiny_layer(seed=0, shape=wl.TINY, cap=64):
    w = wl.layer_weights(shape, seed)
    mats = shape.matrices()
    lw = oracle.LayerWeights(*(oracle.QMat(w[n + ".q"], w[n + ".s"], *mats[n]) for n in ("wqkv", "wo", "wgu", "wdown")),
                             w["norm_attn"], w["norm_ffn"])
    dims = oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn,
                       shape.rms_eps, shape.rope_base, cap)
    return dims, lw


def _empty_cache(dims, slots=1):
    shp = (slots, dims.kv_capacity, dims.n_kv_heads, dims.head_dim)
    return np.full(shp, np.nan, np.float32), np.full(shp, np.nan, np.float32)


def _layer_f64(dims, lw, xbits, K, V, seqs):
    """Independent float64 composition with numpy/scipy library routines (tiny shapes only)."""
    H, h, g, d, F = dims.hidden, dims.n_heads, dims.n_kv_heads, dims.head_dim, dims.ffn
    x = xbits.view(np.float16).astype(np.float64) if xbits.dtype == np.uint16 else np.asarray(xbits, np.float64)
    dq = lambda m: oracle.dequantize(m.q, m.s, m.m, m.k).astype(np.float64)
    nw = lambda b: b.view(np.float16).astype(np.float64)

    def norm(a, w):
        return a / np.sqrt((a * a).mean(axis=1, keepdims=True) + dims.rms_eps) * nw(w)

    qkv = norm(x, lw.norm_attn) @ dq(lw.wqkv).T
    q, k, v = qkv[:, :h * d], qkv[:, h * d:(h + g) * d], qkv[:, (h + g) * d:]
    n = x.shape[0]
    pos = np.concatenate([np.arange(int(seqs.kv[b]) - int(seqs.q[b]), int(seqs.kv[b])) for b in range(len(seqs.q))])
    slot = np.concatenate([np.full(int(seqs.q[b]), b if seqs.sl is None else seqs.sl[b]) for b in range(len(seqs.q))])
    theta = dims.rope_base ** (-2.0 * np.arange(d // 2) / d)

    def rot(a, heads):
        a = a.reshape(n, heads, d).copy()
        ang = pos[:, None, None] * theta[None, None, :]
        lo, hi = a[:, :, :d // 2].copy(), a[:, :, d // 2:].copy()
        a[:, :, :d // 2] = lo * np.cos(ang) - hi * np.sin(ang)
        a[:, :, d // 2:] = lo * np.sin(ang) + hi * np.cos(ang)
        return a

    q, k = rot(q, h), rot(k, g)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for i in range(n):
        K64[slot[i], pos[i]] = k[i]
        V64[slot[i], pos[i]] = v[i].reshape(g, d)
    attn = np.zeros((n, h, d))
    for i in range(n):
        for j in range(h):
            kv = j // (h // g)
            s = K64[slot[i], :pos[i] + 1, kv] @ q[i, j] / np.sqrt(d)
            attn[i, j] = scipy.special.softmax(s) @ V64[slot[i], :pos[i] + 1, kv]
    x1 = x + attn.reshape(n, h * d) @ dq(lw.wo).T
    gu = norm(x1, lw.norm_ffn) @ dq(lw.wgu).T
    act = gu[:, :F] * scipy.special.expit(gu[:, :F]) * gu[:, F:]
    return x1 + act @ dq(lw.wdown).T, K64, V64


def test_layer_against_independent_float64_composition():
    dims, lw = _tiny_layer()
    r = RS(12)
    K, V = _empty_cache(dims, slots=2)
    K[0, :5], V[0, :5] = r.randn(5, 4, 64), r.randn(5, 4, 64)        # sequence 0 has 5 past tokens
    seqs = oracle.Seqs([3, 4], [8, 4], slots=[0, 1])
    x = wl.activations(wl.TINY, 0, 0, 7)
    want, K64, V64 = _layer_f64(dims, lw, x, np.nan_to_num(K), np.nan_to_num(V), seqs)
    out = oracle.decoder_layer(dims, lw, x, K, V, seqs)
    assert np.max(np.abs(out - want)) < 2e-5 * max(1.0, np.max(np.abs(want)))
    assert np.allclose(K[0, :8], K64[0, :8], atol=1e-5) and np.allclose(V[1, :4], V64[1, :4], atol=1e-5)
    assert np.isnan(K[0, 8:]).all() and np.isnan(V[1, 4:]).all()     # nothing written beyond L


def test_layer_zero_projections():
    dims, lw = _tiny_layer()
    x = wl.activations(wl.TINY, 0, 1, 4)
    xf = wl.f16_bits_to_f32(x)
    seqs = oracle.Seqs([4], [4])
    zero = lambda m: oracle.QMat(np.full_like(m.q, 0x88888888), m.s, m.m, m.k)
    lw0 = oracle.LayerWeights(lw.wqkv, zero(lw.wo), lw.wgu, zero(lw.wdown), lw.norm_attn, lw.norm_ffn)
    out = oracle.decoder_layer(dims, lw0, x, *_empty_cache(dims), seqs)
    assert np.array_equal(out.view(np.uint32), xf.view(np.uint32))
    lw1 = oracle.LayerWeights(zero(lw.wqkv), lw.wo, lw.wgu, lw.wdown, lw.norm_attn, lw.norm_ffn)
    out, taps = oracle.decoder_layer(dims, lw1, x, *_empty_cache(dims), seqs, taps=True)
    assert np.all(taps["attn"] == 0) and np.array_equal(taps["x1"], xf)


def test_layer_row_independence_and_prefill_equals_decode_bitwise():
    dims, lw = _tiny_layer()
    n = 6
    x = wl.activations(wl.TINY, 0, 2, n)
    K, V = _empty_cache(dims)
    full = oracle.decoder_layer(dims, lw, x, K, V, oracle.Seqs([n], [n]))
    Ks, Vs = _empty_cache(dims)
    for i in range(n):
        step = oracle.decoder_layer(dims, lw, x[i:i + 1], Ks, Vs, oracle.Seqs([1], [i + 1]))
        assert np.array_equal(step[0].view(np.uint32), full[i].view(np.uint32)), i
    assert np.array_equal(K[0, :n], Ks[0, :n]) and np.array_equal(V[0, :n], Vs[0, :n])
    # ragged batch == each sequence alone
    Kb, Vb = _empty_cache(dims, slots=2)
    both = oracle.decoder_layer(dims, lw, x, Kb, Vb, oracle.Seqs([2, 4], [2, 4]))
    K1, V1 = _empty_cache(dims)
    K2, V2 = _empty_cache(dims)
    a = oracle.decoder_layer(dims, lw, x[:2], K1, V1, oracle.Seqs([2], [2]))
    b = oracle.decoder_layer(dims, lw, x[2:], K2, V2, oracle.Seqs([4], [4]))
    assert np.array_equal(both, np.concatenate([a, b]))


def test_layer_rejects_inconsistent_descriptors():
    dims, lw = _tiny_layer(cap=8)
    x = wl.activations(wl.TINY, 0, 3, 3)
    for q, kv in [([2], [2]), ([3], [2]), ([3], [9]), ([3, 0], [3, 0])]:
        with pytest.raises(ValueError):
            oracle.decoder_layer(dims, lw, x, *_empty_cache(dims, 2), oracle.Seqs(q, kv))


def test_argmax_takes_lowest_index_among_maxima():
    lg = np.array([[0.0, 3.0, 3.0, -1.0], [5.0, 5.0, 5.0, 5.0], [-2.0, -1.0, -3.0, -1.0]], np.float32)
    assert oracle.argmax(lg).tolist() == [1, 0, 1]


# ------------------------------------------------------------------------- model wrapper (Sec. 5.1, end-to-end LLM)
def _tiny_model(n_layers, vocab=97, seed=7, cap=32):
    shape = wl.TINY
    dims = oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.rms_eps, shape.rope_base, cap)
    mats = shape.matrices()
    layers = []
    for l in range(n_layers):
        w = wl.layer_weights(shape, seed, layer=l)
        layers.append(oracle.LayerWeights(*(oracle.QMat(w[n + ".q"], w[n + ".s"], *mats[n]) for n in ("wqkv", "wo", "wgu", "wdown")),
                                          w["norm_attn"], w["norm_ffn"]))
    return shape, dims, layers, wl.model_tensors(shape, seed, vocab)


def _caches(dims, n_layers, slots):
    shp = (slots, dims.kv_capacity, dims.n_kv_heads, dims.head_dim)
    return [np.zeros(shp, np.float32) for _ in range(n_layers)], [np.zeros(shp, np.float32) for _ in range(n_layers)]


def test_model_without_layers_closed_form_and_tied_head_returns_the_input_token():
    shape, dims, _, mt = _tiny_model(0)
    V, H = mt["embedding"].shape
    # (a) constant embedding rows c_v * 1, unit norm weight: y = c/sqrt(c^2+eps) * 1, logits[v'] = y * sum_c W[v',c]
    cvals = (0.25 + 0.125 * np.arange(V)).astype(np.float16)
    emb = np.repeat(cvals[:, None], H, axis=1).view(np.uint16)
    ones = np.ones(H, np.float16).view(np.uint16)
    ids = np.array([3, 50, 96], np.int32)
    logits, _ = oracle.model_step(dims, [], emb, ones, mt["lm_head"], ids, [], [], oracle.Seqs([1, 1, 1], [1, 1, 1]))
    c = cvals[ids].astype(np.float64)
    rowsum = wl.f16_bits_to_f32(mt["lm_head"]).astype(np.float64).sum(axis=1)
    want = (c / np.sqrt(c * c + dims.rms_eps))[:, None] * rowsum[None, :]
    assert np.abs(logits - want).max() < 1e-5
    # (b) LM head tied to a random embedding: <e_id/rms, e_v> is largest at v = id, so greedy returns the input token
    ids = wl.token_ids(7, 9, V)
    _, nxt = oracle.model_step(dims, [], mt["embedding"], ones, mt["embedding"], ids, [], [], oracle.Seqs([1] * 9, [1] * 9))
    assert nxt.tolist() == ids.tolist()


def test_model_reads_the_last_row_of_each_sequence_and_batches_like_separate_calls():
    shape, dims, layers, mt = _tiny_model(2)
    V = mt["embedding"].shape[0]
    ids = wl.token_ids(8, 5 + 1 + 3, V)
    q = [5, 1, 3]
    K, Vc = _caches(dims, 2, 3)
    # sequence 1 is a decode row with 4 cached tokens: give every layer's slot 1 a past
    past = [wl.f16_bits_to_f32(wl.normal_f16_bits(8, 100 + l, (4, dims.n_kv_heads, dims.head_dim))) for l in range(4)]
    for l in range(2):
        K[l][1, :4], Vc[l][1, :4] = past[2 * l], past[2 * l + 1]
    logits, nxt = oracle.model_step(dims, layers, mt["embedding"], mt["norm_final"], mt["lm_head"], ids, K, Vc,
                                    oracle.Seqs(q, [5, 5, 3]))
    assert logits.shape == (3, V) and nxt.shape == (3,)
    # the same three sequences, each in a call of its own (slot 0 of fresh caches)
    start = 0
    for b, (ql, kl) in enumerate(zip(q, [5, 5, 3])):
        Kb, Vb = _caches(dims, 2, 1)
        if b == 1:
            for l in range(2):
                Kb[l][0, :4], Vb[l][0, :4] = past[2 * l], past[2 * l + 1]
        lg, nb = oracle.model_step(dims, layers, mt["embedding"], mt["norm_final"], mt["lm_head"], ids[start:start + ql], Kb, Vb,
                                   oracle.Seqs([ql], [kl]))
        assert np.array_equal(lg[0], logits[b]) and nb[0] == nxt[b]
        # and the layer caches hold the same appended rows
        for l in range(2):
            assert np.array_equal(Kb[l][0, :kl], K[l][b, :kl])
        start += ql
    # a prefill's logits belong to its LAST row: dropping the first rows' successors changes them
    lg_short, _ = oracle.model_step(dims, layers, mt["embedding"], mt["norm_final"], mt["lm_head"], ids[:4], *_caches(dims, 2, 1),
                                    oracle.Seqs([4], [4]))
    assert np.abs(lg_short[0] - logits[0]).max() > 1e-4


def test_model_stack_equals_layer_by_layer_float64_composition():
    """Two layers + head against the float64 layer composition used to pin the single layer."""
    shape, dims, layers, mt = _tiny_model(2, vocab=61)
    ids = wl.token_ids(9, 6, 61)
    K, Vc = _caches(dims, 2, 1)
    logits, _ = oracle.model_step(dims, layers, mt["embedding"], mt["norm_final"], mt["lm_head"], ids, K, Vc, oracle.Seqs([6], [6]))
    x = mt["embedding"][ids]                                    # fp16 bits: the first layer sees exact fp16 values
    seqs = oracle.Seqs([6], [6])
    x64 = None
    for l in range(2):
        zero = np.zeros((1, dims.kv_capacity, dims.n_kv_heads, dims.head_dim))
        x64, _, _ = _layer_f64(dims, layers[l], x if l == 0 else x64, zero, zero.copy(), seqs)
    wf = wl.f16_bits_to_f32(mt["norm_final"]).astype(np.float64)
    last = x64[-1]
    y = last / np.sqrt(np.mean(last * last) + dims.rms_eps) * wf
    want = wl.f16_bits_to_f32(mt["lm_head"]).astype(np.float64) @ y
    assert np.abs(logits[0] - want).max() < 2e-4 * max(1.0, np.abs(want).max())
