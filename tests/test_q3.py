"""3-bit weight format: pins of the CPU reference (hand-derived words, an independent packer, the pinned 4-bit reference
through an exact embedding, a closed form) and, on the GPU, parity of relax_unpack_q3 / relax_dequant_matmul_q3."""
import os

import numpy as np
import pytest

import oracle
from oracle import q3
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "q3_words.txt")


def golden_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                left, right = line.split("=>")
                pos, code = (int(v) for v in left.split())
                cases.append((pos, code, [int(w, 16) for w in right.split()]))
    return cases


@pytest.mark.parametrize("pos,code,words", golden_cases())
def test_hand_derived_words(pos, code, words):
    q = np.array([words], dtype=np.uint32)
    want = np.full((1, 32), -4, dtype=np.int8)
    want[0, pos] = code - 4
    assert np.array_equal(q3.unpack_q3(q, 1, 32), want)
    codes = np.zeros((1, 32), dtype=np.uint8)
    codes[0, pos] = code
    assert np.array_equal(wl.pack_codes3(codes), q)            # the generator's packer agrees with the same hand-derived words


def test_unpack_inverts_the_independent_packer():
    r = np.random.RandomState(5)
    codes = r.randint(0, 8, size=(7, 160)).astype(np.uint8)
    assert np.array_equal(q3.unpack_q3(wl.pack_codes3(codes), 7, 160), codes.astype(np.int8) - 4)


def test_matmul_equals_the_4bit_reference_on_embedded_codes():
    # u3 - 4 == (u3 + 4) - 8: the same matrix written as 4-bit codes must give the pinned 4-bit reference's product
    m, k, n = 9, 96, 3
    r = np.random.RandomState(6)
    codes = r.randint(0, 8, size=(m, k)).astype(np.uint8)
    s = (r.rand(m, k // 32) * 0.02 + 0.001).astype(np.float16).view(np.uint16)
    x = r.randn(n, k).astype(np.float32)
    ref4 = oracle.dequant_matmul(x, wl.pack_codes(codes + 4), s, m, k)
    got = q3.dequant_matmul_q3(x, wl.pack_codes3(codes), s, m, k)
    assert np.abs(got - ref4).max() <= 1e-5 * max(1.0, np.abs(ref4).max())
    assert np.array_equal(q3.dequantize_q3(wl.pack_codes3(codes), s, m, k).astype(np.float32), oracle.dequantize(wl.pack_codes(codes + 4), s, m, k))


def test_closed_form():
    m, k = 4, 64
    q = wl.pack_codes3(np.full((m, k), 7, dtype=np.uint8))                 # every weight 3 * 0.5
    s = np.full((m, k // 32), np.float16(0.5)).view(np.uint16)
    assert np.array_equal(q3.dequant_matmul_q3(np.ones((2, k), np.float32), q, s, m, k), np.full((2, m), 1.5 * k))


def test_quantiser_stays_in_range_and_close():
    w = wl.rng(3, 1).standard_normal((5, 64), dtype=np.float32) * np.float32(0.02)
    q, s = wl.quantize_q3(w)
    codes = q3.unpack_q3(q, 5, 64)
    assert codes.min() >= -3 and codes.max() <= 3
    step = np.repeat(s.view(np.float16).astype(np.float64), 32, axis=1)
    assert np.all(np.abs(q3.dequantize_q3(q, s, 5, 64) - w) <= 0.5 * step + 1e-6)


def test_layer_equals_the_4bit_reference_layer_on_embedded_codes():
    """The composed 3-bit layer reference against the C reference of the 4-bit layer on the same real matrices
    (u3 - 4 == (u3 + 4) - 8, same scales): a prefill of 5 rows and two decode steps, caches included."""
    from helpers import oracle_dims
    shape = wl.LayerShape("q3-pin", hidden=64, n_heads=2, n_kv_heads=1, head_dim=32, ffn=96)
    r = np.random.RandomState(11)
    w3, w4 = {}, {}
    for name, (m, k) in shape.matrices().items():
        codes = r.randint(0, 8, size=(m, k)).astype(np.uint8)
        sc = (r.rand(m, k // 32) * 0.05 + 0.01).astype(np.float16).view(np.uint16)
        w3[name + ".q"], w3[name + ".s"] = wl.pack_codes3(codes), sc
        w4[name + ".q"], w4[name + ".s"] = wl.pack_codes(codes + 4), sc
    for name in ("norm_attn", "norm_ffn"):
        w3[name] = w4[name] = wl.normal_f16_bits(11, 7 if name == "norm_attn" else 8, (shape.hidden,), std=0.1, mean=1.0)
    od = oracle_dims(shape, 16)
    ow4 = oracle.LayerWeights(*(oracle.QMat(w4[n_ + ".q"], w4[n_ + ".s"], *shape.matrices()[n_]) for n_ in ("wqkv", "wo", "wgu", "wdown")),
                              w4["norm_attn"], w4["norm_ffn"])
    cs = (1, 16, shape.n_kv_heads, shape.head_dim)
    K3, V3, K4, V4 = (np.zeros(cs, np.float32) for _ in range(4))
    for ci, (ql, kl) in enumerate([([5], [5]), ([1], [6]), ([1], [7])]):
        x = wl.activations(shape, 11, ci, ql[0])
        ref = oracle.decoder_layer(od, ow4, x, K4, V4, oracle.Seqs(ql, kl, None))
        got = q3.decoder_layer_q3(od, w3, x, K3, V3, oracle.Seqs(ql, kl, None))
        assert np.abs(got - ref).max() <= 2e-5 * max(1.0, np.abs(ref).max()), ci
    assert np.abs(K3 - K4).max() <= 1e-5 and np.abs(V3 - V4).max() <= 1e-5


# ------------------------------------------------------------------------------------------------ GPU parity
@pytest.fixture(scope="module")
def rx():
    from paper_2311_02103_amd import binding
    binding.lib()
    return binding


def gpu_q3_matmul(rx, x_bits, q, s, m, k):
    import torch
    n = x_bits.shape[0]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int32 if a.dtype == np.uint32 else np.int16)).cuda()
    out = torch.empty((n, m), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_dequant_matmul_q3(dev(x_bits), rx.QMat(dev(q), dev(s), m, k), out, n), "relax_dequant_matmul_q3")
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float32)


@pytest.mark.gpu
@pytest.mark.parametrize("m,k", [(1, 32), (5, 96), (33, 704), (64, 4096), (3, 11008)])
def test_gpu_unpack_bit_exact(rx, m, k):
    import torch
    r = np.random.RandomState(m * 7 + k)
    q = r.randint(0, 2 ** 32, size=(m, 3 * k // 32), dtype=np.uint64).astype(np.uint32)
    qd = torch.from_numpy(q.view(np.int32)).cuda()
    out = torch.empty((m, k), dtype=torch.int8, device="cuda")
    rx.check(rx.relax_unpack_q3(rx.QMat(qd, qd, m, k), out), "relax_unpack_q3")
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), q3.unpack_q3(q, m, k))


@pytest.mark.gpu
@pytest.mark.parametrize("m,k,n", [(40, 256, 2), (65, 704, 3), (130, 4096, 1), (37, 11008, 2)])
def test_gpu_integer_valued_matmul_bitwise(rx, m, k, n):
    """Random codes, scales 1 and 2, sparse small-integer x: every partial sum is an integer below 2^24 and the result is at
    most 2048 in magnitude, so the fp16 output must equal the reference exactly — any slip in word, bit offset, straddling
    code or scale group shows as a wrong integer."""
    r = np.random.RandomState(k + m)
    codes = r.randint(0, 8, size=(m, k)).astype(np.uint8)
    s = r.choice([1.0, 2.0], size=(m, k // 32)).astype(np.float16).view(np.uint16)
    x = np.zeros((n, k), dtype=np.float32)
    hot = r.choice(k, size=40, replace=False)
    x[:, hot] = r.randint(-3, 4, size=(n, 40))
    q = wl.pack_codes3(codes)
    ref = q3.dequant_matmul_q3(x, q, s, m, k)
    assert np.abs(ref).max() <= 2048
    got = gpu_q3_matmul(rx, x.astype(np.float16).view(np.uint16), q, s, m, k)
    assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.gpu
@pytest.mark.parametrize("m,k,n", [(1, 32, 1), (7, 64, 3), (257, 704, 1), (1000, 2048 + 32, 5), (4099, 4096, 1), (22016, 4096, 1),
                                   (4096, 11008, 2), (300, 12288, 1), (515, 4096, 17)])
def test_gpu_matmul_random(rx, m, k, n):
    """Quantised N(0, 0.02^2) weights, N(0,1) x: ragged m, every groups-per-lane variant of the kernel (k from 32 to
    12288), several rows of x."""
    q, s = wl.qmat3(8, m * 131 + k, m, k)
    x = wl.normal_f16_bits(8, m + k + n, (n, k))
    ref = q3.dequant_matmul_q3(wl.f16_bits_to_f32(x), q, s, m, k)
    got = gpu_q3_matmul(rx, x, q, s, m, k)
    err = np.abs(got - ref)
    assert np.all(err <= 1e-2 + 2e-2 * np.abs(ref)), "m=%d k=%d n=%d: max err %g" % (m, k, n, err.max())
    assert err.max() <= 2e-3 * max(1.0, np.abs(ref).max())


# ------------------------------------------------------------------------------------------------ GPU-native layout
def gpu_q3_native(rx, q):
    """canonical words on the host -> native words on the device (relax_repack_q3)"""
    import torch
    m, w = q.shape
    qd = torch.from_numpy(q.view(np.int32)).cuda()
    nat = torch.empty_like(qd)
    rx.check(rx.relax_repack_q3(rx.QMat(qd, qd, m, w * 32 // 3), nat), "relax_repack_q3")
    return nat


def gpu_q3_native_matmul(rx, x_bits, q, s, m, k):
    import torch
    n = x_bits.shape[0]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a).view(np.int32 if a.dtype == np.uint32 else np.int16)).cuda()
    out = torch.full((n, m), float("nan"), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_dequant_matmul_q3_native(dev(x_bits), rx.QMat(gpu_q3_native(rx, q), dev(s), m, k), out, n), "relax_dequant_matmul_q3_native")
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float32)


@pytest.mark.gpu
@pytest.mark.parametrize("m,k", [(1, 32), (5, 96), (33, 704), (64, 4096), (3, 11008)])
def test_gpu_repack_then_native_unpack_bit_exact(rx, m, k):
    """Random words (every code at every position, both straddling codes): the native layout decodes to what the canonical
    one decodes to, element by element."""
    import torch
    r = np.random.RandomState(m * 11 + k)
    q = r.randint(0, 2 ** 32, size=(m, 3 * k // 32), dtype=np.uint64).astype(np.uint32)
    nat = gpu_q3_native(rx, q)
    out = torch.empty((m, k), dtype=torch.int8, device="cuda")
    rx.check(rx.relax_unpack_q3_native(rx.QMat(nat, nat, m, k), out), "relax_unpack_q3_native")
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), q3.unpack_q3(q, m, k))
    # one code set at a time: the native word image is what the layout's definition says (column -> word, bit)
    codes = np.zeros((32, 32), dtype=np.uint8)
    codes[np.arange(32), np.arange(32)] = 5                       # row c: u_c = 5 (binary 101), all other codes 0
    nat = gpu_q3_native(rx, wl.pack_codes3(codes)).cpu().numpy().view(np.uint32)
    want = np.zeros((32, 3), dtype=np.uint32)
    for c in range(30):
        p = c // 2
        want[c, p // 5] = 5 << (3 * (p % 5) + 16 * (c % 2))
    for c in (30, 31):
        want[c, 0] = want[c, 2] = 1 << (15 if c == 30 else 31)    # bits 0 and 2 of the code go to words 0 and 2
    assert np.array_equal(nat, want)


@pytest.mark.gpu
@pytest.mark.parametrize("m,k,n", [(40, 256, 2), (65, 704, 3), (130, 4096, 1), (131, 4096, 4), (37, 11008, 2), (64, 8192, 5)])
def test_gpu_native_integer_valued_matmul_bitwise(rx, m, k, n):
    r = np.random.RandomState(k + m + n)
    codes = r.randint(0, 8, size=(m, k)).astype(np.uint8)
    s = r.choice([1.0, 2.0], size=(m, k // 32)).astype(np.float16).view(np.uint16)
    x = np.zeros((n, k), dtype=np.float32)
    hot = r.choice(k, size=40, replace=False)
    x[:, hot] = r.randint(-3, 4, size=(n, 40))
    q = wl.pack_codes3(codes)
    ref = q3.dequant_matmul_q3(x, q, s, m, k)
    assert np.abs(ref).max() <= 2048
    got = gpu_q3_native_matmul(rx, x.astype(np.float16).view(np.uint16), q, s, m, k)
    assert np.array_equal(got.astype(np.float64), ref)


@pytest.mark.gpu
@pytest.mark.parametrize("m,k,n", [(1, 32, 1), (7, 64, 3), (257, 704, 1), (1000, 2048 + 32, 5), (4099, 4096, 1), (22016, 4096, 1),
                                   (4096, 11008, 2), (300, 12288, 1), (515, 4096, 17), (1001, 8192, 7), (333, 6144, 4)])
def test_gpu_native_matmul_random(rx, m, k, n):
    """Every (groups per lane, rows per pass) variant of the native-layout kernel, odd m, ragged last passes."""
    q, s = wl.qmat3(9, m * 131 + k, m, k)
    x = wl.normal_f16_bits(9, m + k + n, (n, k))
    ref = q3.dequant_matmul_q3(wl.f16_bits_to_f32(x), q, s, m, k)
    got = gpu_q3_native_matmul(rx, x, q, s, m, k)
    err = np.abs(got - ref)
    assert np.all(err <= 1e-2 + 2e-2 * np.abs(ref)), "m=%d k=%d n=%d: max err %g" % (m, k, n, err.max())
    assert err.max() <= 2e-3 * max(1.0, np.abs(ref).max())


# From 16 rows of x on, a matrix with k % 128 == 0 and m % 4 == 0 goes through the tiled MFMA GEMM (3-bit decode on the way
# into LDS); every tile shape of it is met below (n <= 64: 128 x 64; <= 128: 128 x 128; above: 128 x 256 and 256 x 256).
@pytest.mark.gpu
@pytest.mark.parametrize("m,k,n", [(128, 256, 16), (64, 4096, 40), (260, 1024, 100), (512, 2048, 200), (1024, 1024, 300), (96, 16384, 17)])
def test_gpu_native_gemm_integer_valued_bitwise(rx, m, k, n):
    r = np.random.RandomState(k + m + n)
    codes = r.randint(0, 8, size=(m, k)).astype(np.uint8)
    s = r.choice([1.0, 2.0], size=(m, k // 32)).astype(np.float16).view(np.uint16)
    x = np.zeros((n, k), dtype=np.float32)
    hot = r.choice(k, size=40, replace=False)
    x[:, hot] = r.randint(-3, 4, size=(n, 40))
    q = wl.pack_codes3(codes)
    ref = q3.dequant_matmul_q3(x, q, s, m, k)
    assert np.abs(ref).max() <= 2048 and np.abs(ref).max() > 0
    got = gpu_q3_native_matmul(rx, x.astype(np.float16).view(np.uint16), q, s, m, k)
    assert np.array_equal(got.astype(np.float64), ref)
    # a selector matrix (one code 5 = +1 per row, all others 4 = 0, scale 1) picks integer-valued x exactly: a wrong column
    # order inside a group, or between the weight tile and the x tile, picks the wrong element
    codes = np.full((m, k), 4, dtype=np.uint8)
    cols = (7 * np.arange(m) + 3) % k
    codes[np.arange(m), cols] = 5
    xi = ((np.arange(n)[:, None] * 5 + np.arange(k)[None, :] * 37) % 15 - 7).astype(np.float32)
    ones = np.full((m, k // 32), np.float16(1.0)).view(np.uint16)
    got = gpu_q3_native_matmul(rx, xi.astype(np.float16).view(np.uint16), wl.pack_codes3(codes), ones, m, k)
    assert np.array_equal(got, xi[:, cols])


@pytest.mark.gpu
@pytest.mark.parametrize("m,k,n", [(512, 4096, 16), (1000, 2048, 300), (4096, 4096, 128), (22016, 4096, 64), (4096, 11008, 130), (256, 16384, 33),
                                   (12288, 4096, 511)])
def test_gpu_native_gemm_random(rx, m, k, n):
    q, s = wl.qmat3(9, m * 131 + k, m, k)
    x = wl.normal_f16_bits(9, m + k + n, (n, k))
    ref = q3.dequant_matmul_q3(wl.f16_bits_to_f32(x), q, s, m, k)
    got = gpu_q3_native_matmul(rx, x, q, s, m, k)
    err = np.abs(got - ref)
    assert np.all(err <= 1e-2 + 2e-2 * np.abs(ref)), "m=%d k=%d n=%d: max err %g" % (m, k, n, err.max())
    assert err.max() <= 3e-3 * max(1.0, np.abs(ref).max())


def test_host_checks_of_the_q3_entry_points():
    from paper_2311_02103_amd import binding as rx
    if not os.path.exists(rx.LIB_PATH):
        pytest.skip("library not built")
    w = rx.QMatC(64, 64, 8, 64, 32)                # non-NULL fake pointers: every case below is rejected before any launch
    assert rx.lib().relax_dequant_matmul_q3(None, w, 64, 1, None) == rx.ERR_NULL
    assert rx.lib().relax_dequant_matmul_q3(64, w, 64, 0, None) == rx.ERR_SHAPE
    assert rx.lib().relax_dequant_matmul_q3(64, rx.QMatC(64, 64, 8, 40), 64, 1, None) == rx.ERR_SHAPE          # k % 32
    assert rx.lib().relax_dequant_matmul_q3(64, rx.QMatC(64, 64, 8, 12288 + 32), 64, 1, None) == rx.ERR_UNSUPPORTED
    assert rx.lib().relax_dequant_matmul_q3(72, w, 64, 1, None) == rx.ERR_SHAPE                                 # x not 16-byte aligned
    assert rx.lib().relax_unpack_q3(None, 64, None) == rx.ERR_NULL
    assert rx.lib().relax_unpack_q3(rx.QMatC(64, 64, 8, 48), 64, None) == rx.ERR_SHAPE
    assert rx.lib().relax_repack_q3(None, 64, None) == rx.ERR_NULL
    assert rx.lib().relax_repack_q3(w, 64, None) == rx.ERR_SHAPE                                               # in place
    assert rx.lib().relax_repack_q3(rx.QMatC(64, 64, 8, 40), 128, None) == rx.ERR_SHAPE
    assert rx.lib().relax_unpack_q3_native(rx.QMatC(64, 64, 8, 48), 64, None) == rx.ERR_SHAPE
    assert rx.lib().relax_dequant_matmul_q3_native(64, w, 64, 0, None) == rx.ERR_SHAPE
    assert rx.lib().relax_dequant_matmul_q3_native(64, rx.QMatC(64, 64, 8, 12288 + 32), 64, 1, None) == rx.ERR_UNSUPPORTED    # one row: matvec only
    assert rx.lib().relax_dequant_matmul_q3_native(None, w, 64, 1, None) == rx.ERR_NULL


# ------------------------------------------------------------------------------------------------ the layer on 3-bit weights
Q3_SMALL = wl.LayerShape("q3-small", hidden=256, n_heads=4, n_kv_heads=2, head_dim=64, ffn=704)
Q3_MID = wl.LayerShape("q3-mid", hidden=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn=5632)


def run_q3_schedule(rx, shape, seed, cap, calls, slots=1):
    import torch
    from helpers import assert_close, oracle_dims
    from paper_2311_02103_amd.runtime import DeviceLayerQ3, f16_bits, to_device
    w = wl.layer_weights3(shape, seed)
    n_max = max(int(np.sum(c[0])) for c in calls)
    layer = DeviceLayerQ3(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                          ffn=shape.ffn, kv_capacity=cap, kv_slots=slots, n_max=n_max, B_max=max(len(c[0]) for c in calls),
                          rms_eps=shape.rms_eps, rope_base=shape.rope_base)
    od = oracle_dims(shape, cap)
    cshape = (slots, cap, shape.n_kv_heads, shape.head_dim)
    Ko, Vo = np.zeros(cshape, np.float32), np.zeros(cshape, np.float32)
    for ci, (ql, kl, sl) in enumerate(calls):
        n = int(np.sum(ql))
        x = wl.activations(shape, seed, ci, n)
        y = layer.forward(to_device(x), ql, kl, sl)
        torch.cuda.synchronize()
        ref = q3.decoder_layer_q3(od, w, x, Ko, Vo, oracle.Seqs(ql, kl, sl))
        assert_close(f16_bits(y).view(np.float16).astype(np.float32), ref, "%s 3-bit layer, call %d (n = %d)" % (shape.name, ci, n))
    Kg, Vg = f16_bits(layer.k).view(np.float16).astype(np.float32), f16_bits(layer.v).view(np.float16).astype(np.float32)
    assert_close(Kg.reshape(cshape), Ko, "K cache", atol=5e-3, rtol=5e-3)
    assert_close(Vg.reshape(cshape), Vo, "V cache", atol=5e-3, rtol=5e-3)


@pytest.mark.gpu
def test_gpu_q3_layer_small_prefill_decode_and_ragged_batch(rx):
    """Grouped heads, k = 256 and 704: a prefill (rows through the matvec passes: 704 is not a multiple of 128), decode steps,
    a ragged batch over three slots."""
    calls = [([21], [21], [0]), ([1], [22], [0]), ([1], [23], [0]), ([3, 1, 5], [3, 24, 5], [1, 0, 2]), ([1, 1, 1], [4, 25, 6], [1, 0, 2])]
    run_q3_schedule(rx, Q3_SMALL, 13, 40, calls, slots=3)


@pytest.mark.gpu
def test_gpu_q3_layer_mid_through_matvec_and_gemm(rx):
    """k = 2048 and 5632: one decode row and a few rows through the matvec passes, 40 and 130 rows through the tiled GEMM."""
    calls = [([40], [40], None), ([1], [41], None), ([3], [44], None), ([130], [174], None), ([1], [175], None)]
    run_q3_schedule(rx, Q3_MID, 17, 192, calls)


def test_host_checks_of_the_q3_layer():
    from paper_2311_02103_amd import binding as rx
    if not os.path.exists(rx.LIB_PATH):
        pytest.skip("library not built")
    dims = rx.make_dims(256, 4, 2, 64, 704, 32, 1, 1e-5, 10000.0, 32)
    assert rx.relax_layer_q3_workspace_bytes(dims, 8, 32, 2) > 0
    assert rx.relax_layer_q3_workspace_bytes(None, 8, 32, 2) == 0
    assert rx.relax_layer_q3_workspace_bytes(dims, 0, 32, 2) == 0
    assert rx.relax_layer_q3_workspace_bytes(dims, 16, 32, 2) > rx.relax_layer_q3_workspace_bytes(dims, 8, 32, 2)
    assert rx.relax_decoder_layer_q3(dims, None, 64, None, None, 64, 1, 256, 1 << 20) == rx.ERR_NULL


@pytest.mark.gpu
def test_gpu_q3_layer_7b_shape_decode_rows(rx):
    """The 7B layer shape (k = 4096 and 11008: the two- and six-chunk variants of the fused one-row path, attention merge
    folded into the output projection): a short prefill, then two decode rows."""
    calls = [([6], [6], None), ([1], [7], None), ([1], [8], None)]
    run_q3_schedule(rx, wl.LLAMA7B, 19, 64, calls)


@pytest.mark.gpu
def test_gpu_q3_layer_hidden_5120_decode_rows(rx):
    """Hidden width of the 13B shape (2.5 chunks of 2048 columns: the three-chunk variants of the fused one-row path, merge
    folded in): a short prefill, then two decode rows."""
    shape = wl.LayerShape("q3-h5120", hidden=5120, n_heads=40, n_kv_heads=40, head_dim=128, ffn=1024)
    run_q3_schedule(rx, shape, 23, 32, [([4], [4], None), ([1], [5], None), ([1], [6], None)])
