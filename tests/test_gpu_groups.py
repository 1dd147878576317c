"""Quantisation groups of 64 and 128 columns through the C ABI, against the oracle (whose group generalisation is pinned
on the CPU in test_oracle_pins.py): decode exports bit-exact, exact matmul cases bitwise on every kernel that takes such a
matrix (the x-in-registers matvec, the LDS-resident matvec for long rows, the word-by-word matvec for k % 32 != 0, the
few-row split-K kernel, the tiled MFMA GEMM), random matmuls and whole layers within the fp16 bar."""
import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import assert_close, f32_cache, oracle_dims
from test_gpu_parity import dev, gpu_matmul, host_bits

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
GROUPS = [64, 128]


@pytest.fixture(scope="module")
def rx():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2311_02103_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("m,k", [(5, 64), (33, 688), (64, 4096), (3, 11008)])
def test_dequantize_bit_exact(rx, m, k, group):
    r = np.random.RandomState(m * 7 + k + group)
    q = r.randint(0, 2 ** 32, size=(m, k // 8), dtype=np.uint64).astype(np.uint32)           # all 16 codes
    s = (r.randn(m, (k + group - 1) // group) * 0.01).astype(np.float16).view(np.uint16)
    dense = torch.empty((m, k), dtype=torch.float32, device="cuda")
    rx.check(rx.relax_dequantize(rx.QMat(dev(q), dev(s), m, k, group), dense), "relax_dequantize")
    torch.cuda.synchronize()
    assert np.array_equal(dense.cpu().numpy().view(np.uint32), oracle.dequantize(q, s, m, k, group).view(np.uint32))


# n: 1 = matvec kernels; 3 = few-row kernel (k % 256 == 0, with a workspace) or matvec passes; 16.. = few-row kernel or tiled MFMA GEMM
@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("m,k,n", [(130, 4096, 1), (37, 11008, 1), (65, 688, 1), (12, 16384, 1), (40, 256, 3), (64, 4096, 3),
                                   (128, 4096, 16), (256, 1024, 200), (96, 11008, 64), (132, 2048, 7), (260, 8192, 33), (128, 1024, 100)])
def test_exact_cases_bitwise(rx, m, k, n, group):
    """Per-group scales are distinct powers of two and codes random, x sparse small integers: every output is an integer
    that fp16 holds exactly, so a wrong scale index (sub-group -> scale, row stride ceil(k / group)) shows as a wrong
    integer.  Then a selector matrix with scale 1."""
    r = np.random.RandomState(k + m + group)
    SG = (k + group - 1) // group
    codes = r.randint(0, 16, size=(m, k)).astype(np.uint8)
    sc = np.ldexp(1.0, (np.arange(SG)[None, :] + np.arange(m)[:, None]) % 3).astype(np.float16)    # 1, 2, 4 by (row, group)
    x = np.zeros((n, k), dtype=np.float32)
    hot = r.choice(k, size=16, replace=False)
    x[:, hot] = r.randint(-2, 3, size=(n, 16))
    q, s = wl.pack_codes(codes), sc.view(np.uint16)
    ref = oracle.dequant_matmul(x, q, s, m, k, group)
    assert np.abs(ref).max() <= 2048 and np.abs(ref).max() > 0
    for with_ws in (False, True):               # with a workspace 2..128 rows take the few-row split-K kernel
        got = gpu_matmul(rx, x.astype(np.float16).view(np.uint16), q, s, m, k, with_ws=with_ws, group=group).view(np.float16).astype(np.float32)
        assert np.array_equal(got, ref), with_ws
    codes = np.full((m, k), 8, dtype=np.uint8)
    cols = (7 * np.arange(m) + 3) % k
    codes[np.arange(m), cols] = 9
    xi = ((np.arange(n)[:, None] * 5 + np.arange(k)[None, :] * 37) % 15 - 7).astype(np.float32)
    ones = np.full((m, SG), np.float16(1.0)).view(np.uint16)
    got = gpu_matmul(rx, xi.astype(np.float16).view(np.uint16), wl.pack_codes(codes), ones, m, k, group=group).view(np.float16).astype(np.float32)
    assert np.array_equal(got, xi[:, cols])


@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("m,k,n", [(1024, 4096, 1), (640, 11008, 1), (257, 688, 1), (2, 28672, 1), (131, 2080, 1), (515, 4096, 5),
                                   (768, 256, 37), (4096, 4096, 128), (1000, 2048, 300)])
def test_random_matmul(rx, m, k, n, group):
    q, s = wl.qmat(50, m * 131 + k + group, m, k, group=group)
    x = wl.normal_f16_bits(50, m + k + n, (n, k))
    ref = oracle.dequant_matmul(wl.f16_bits_to_f32(x), q, s, m, k, group)
    for with_ws in (False, True):
        got = gpu_matmul(rx, x, q, s, m, k, with_ws=with_ws, group=group).view(np.float16).astype(np.float32)
        assert_close(got, ref, "group %d m=%d k=%d n=%d" % (group, m, k, n))
        assert np.abs(got - ref).max() <= 3e-3 * max(1.0, np.abs(ref).max())


MID = wl.LayerShape("mid-mha", hidden=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn=5632)
MID_GQA = wl.LayerShape("mid-gqa", hidden=1024, n_heads=16, n_kv_heads=4, head_dim=64, ffn=2816)


@pytest.mark.parametrize("group", GROUPS)
@pytest.mark.parametrize("shape,calls", [
    (wl.TINY, [([9], [9], None), ([1], [10], None)]),                               # k = 688: short last group (48 of 64, 48 of 128)
    (MID, [([40], [40], None), ([1], [41], None), ([3], [44], None), ([200], [244], None)]),   # few-row kernel, matvec, few-row kernel, GEMM
    (MID_GQA, [([5, 1, 20], [5, 1, 20], [2, 0, 1]), ([1, 1, 1], [6, 2, 21], [2, 0, 1])]),
])
def test_layer_with_wider_groups(rx, shape, calls, group):
    from paper_2311_02103_amd.runtime import DeviceLayer
    cap, slots = 256, 3
    w = wl.layer_weights(shape, 60 + group, group=group)
    n_max = max(int(np.sum(c[0])) for c in calls)
    layer = DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                        ffn=shape.ffn, kv_capacity=cap, kv_slots=slots, n_max=n_max, B_max=slots, group=group)
    mats = shape.matrices()
    ow = oracle.LayerWeights(*(oracle.QMat(w[nm + ".q"], w[nm + ".s"], *mats[nm], group) for nm in ("wqkv", "wo", "wgu", "wdown")),
                             w["norm_attn"], w["norm_ffn"])
    od = oracle_dims(shape, cap)
    Ko = np.zeros((slots, cap, shape.n_kv_heads, shape.head_dim), np.float32)
    Vo = np.zeros_like(Ko)
    for ci, (ql, kl, sl) in enumerate(calls):
        n = int(np.sum(ql))
        x = wl.activations(shape, 60, ci, n)
        y = layer.forward(dev(x), ql, kl, sl)
        torch.cuda.synchronize()
        ref = oracle.decoder_layer(od, ow, x, Ko, Vo, oracle.Seqs(ql, kl, sl))
        assert_close(host_bits(y).view(np.float16).astype(np.float32), ref, "%s group %d call %d" % (shape.name, group, ci))
    assert_close(host_bits(layer.k).view(np.float16).astype(np.float32), Ko, "K cache", atol=5e-3, rtol=5e-3)
