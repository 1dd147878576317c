"""Randomised ragged calls of relax_decoder_layer against the oracle: decode batches, ragged prefills and mixtures, with
the descriptor on the host or in a device table (host bounds loose), random slots and cached lengths, on mid-size
shapes whose matrices take every dispatch path (matvec kernels, few-row kernel, tiled GEMM with and without k splits)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import assert_close, oracle_dims, oracle_weights, f32_cache

pytestmark = pytest.mark.gpu

SHAPES = [wl.LayerShape("mid-mha", hidden=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn=5632),
          wl.LayerShape("mid-gqa", hidden=2048, n_heads=32, n_kv_heads=4, head_dim=64, ffn=5632),
          wl.LayerShape("odd-gqa", hidden=1024, n_heads=8, n_kv_heads=2, head_dim=128, ffn=2816)]


@pytest.fixture(scope="module")
def rx():
    from paper_2311_02103_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("si", range(len(SHAPES)))
def test_random_ragged_calls_against_the_oracle(rx, si):
    from paper_2311_02103_amd.runtime import DeviceLayer
    shape, cap, slots, n_max = SHAPES[si], 200, 24, 300
    rng = np.random.default_rng(1000 + si)
    w = wl.layer_weights(shape, 50 + si)
    layer = DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                        ffn=shape.ffn, kv_capacity=cap, kv_slots=slots, n_max=n_max, B_max=slots)
    od, ow = oracle_dims(shape, cap), oracle_weights(shape, w)
    kb, vb = wl.kv_prefill(shape, 60 + si, slots, cap)
    cshape = (slots, cap, shape.n_kv_heads, shape.head_dim)
    for it in range(9):
        B = int(rng.choice([1, 2, 3, 5, 17, 20]))
        mode = ["decode", "prefill", "mixed"][it % 3]
        if mode == "decode":
            q = [1] * B
        elif mode == "prefill":
            q = [int(rng.integers(1, 140)) for _ in range(B)]
        else:
            q = [int(rng.choice([1, 1, int(rng.integers(2, 40))])) for _ in range(B)]
        while sum(q) > n_max:
            q[int(np.argmax(q))] //= 2
        q = [max(1, v) for v in q]
        kv = [int(rng.integers(v, cap + 1)) for v in q]
        sl = [int(v) for v in rng.permutation(slots)[:B]]
        n = sum(q)
        layer.load_cache(kb, vb)
        Ko, Vo = f32_cache(kb).reshape(cshape).copy(), f32_cache(vb).reshape(cshape).copy()
        x = wl.activations(shape, 70 + si, it, n)
        xt = torch.from_numpy(x.view(np.int16)).view(torch.float16).cuda()
        what = "%s call %d (%s, n=%d, B=%d, q=%s, kv=%s, slots=%s)" % (shape.name, it, mode, n, B, q, kv, sl)
        if it % 2:                                                 # descriptor on the device, capacity as the host bound
            starts = np.concatenate([[0], np.cumsum(q)[:-1]])
            tab = torch.from_numpy(np.stack([starts, q, kv, sl]).astype(np.int32)).cuda().contiguous()
            y = layer.forward(xt, q, [cap] * B, None, device_table=tab)
        else:
            y = layer.forward(xt, q, kv, sl)
        torch.cuda.synchronize()
        ref = oracle.decoder_layer(od, ow, x, Ko, Vo, oracle.Seqs(q, kv, sl))
        assert_close(y.float().cpu().numpy(), ref, what)
        assert_close(layer.k.float().cpu().numpy(), Ko, what + ": K cache", atol=5e-3, rtol=5e-3)
        assert_close(layer.v.float().cpu().numpy(), Vo, what + ": V cache", atol=5e-3, rtol=5e-3)


def test_70b_shape_ragged_calls_against_the_oracle(rx):
    """The same at the 70B layer shape (hidden 8192, 64 query / 8 KV heads, ffn 28672): matvec, few-row and tiled-GEMM
    calls, decode rows, chunked and fresh prefills.  With synthetic weights of fixed RMS 0.03 the down projection sums
    28672 terms and the layer output has RMS 7.6, so elements where that sum cancels carry the rounding noise of the
    whole sum: the absolute part of the tolerance is taken relative to the RMS of the reference output (as for logits),
    and the RMS of the error itself must stay at the level fp16 intermediates explain (observed 0.4e-3 at n = 1 to
    1.5e-3 of the output RMS on long prefills, whose later rows attend to K/V the call itself rounded to fp16)."""
    from paper_2311_02103_amd.runtime import DeviceLayer
    shape, cap, slots, n_max = wl.LLAMA70B, 2048, 5, 600
    w = wl.layer_weights(shape, 250)
    layer = DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                        ffn=shape.ffn, kv_capacity=cap, kv_slots=slots, n_max=n_max, B_max=slots)
    od, ow = oracle_dims(shape, cap), oracle_weights(shape, w)
    kb, vb = wl.kv_prefill(shape, 260, slots, cap)
    cshape = (slots, cap, shape.n_kv_heads, shape.head_dim)
    calls = [([1], [1286], [3]),                                             # matvec kernels
             ([1, 1, 1, 1], [1789, 1383, 307, 1125], [1, 0, 2, 4]),            # few-row kernel, grouped-query decode attention
             ([1, 23, 1, 16], [563, 1005, 568, 16], [4, 0, 2, 1]),             # few-row kernel, mixed rows
             ([115, 103, 178, 102], [1604, 163, 745, 793], [4, 1, 0, 3]),      # tiled GEMM, chunked prefills
             ([241, 199, 128], [241, 2048, 128], [3, 1, 2]),                   # tiled GEMM, fresh prefills and a full cache
             ([1, 1], [907, 1466], [2, 0]),                                    # two decode rows: matvec kernels, two rows of x per pass
             ([1, 1], [33, 2048], [1, 4])]                                     # the same through the device table
    for it, (q, kv, sl) in enumerate(calls):
        n, B = sum(q), len(q)
        layer.load_cache(kb, vb)
        Ko, Vo = f32_cache(kb).reshape(cshape).copy(), f32_cache(vb).reshape(cshape).copy()
        x = wl.activations(shape, 270, it, n)
        xt = torch.from_numpy(x.view(np.int16)).view(torch.float16).cuda()
        what = "70B shape call %d (n=%d, q=%s, kv=%s, slots=%s)" % (it, n, q, kv, sl)
        if it % 2:
            starts = np.concatenate([[0], np.cumsum(q)[:-1]])
            tab = torch.from_numpy(np.stack([starts, q, kv, sl]).astype(np.int32)).cuda().contiguous()
            y = layer.forward(xt, q, [cap] * B, None, device_table=tab)
        else:
            y = layer.forward(xt, q, kv, sl)
        torch.cuda.synchronize()
        ref = oracle.decoder_layer(od, ow, x, Ko, Vo, oracle.Seqs(q, kv, sl))
        got = y.float().cpu().numpy()
        ref_rms = float(np.sqrt(np.mean(np.square(ref, dtype=np.float64))))
        err_rms = float(np.sqrt(np.mean(np.square(got.astype(np.float64) - ref))))
        assert 5.0 < ref_rms < 12.0, (what, ref_rms)
        assert_close(got, ref, what, atol=1e-2 * ref_rms)
        assert err_rms <= 2.5e-3 * ref_rms, "%s: error RMS %.3e against output RMS %.3f" % (what, err_rms, ref_rms)
        assert_close(layer.k.float().cpu().numpy(), Ko, what + ": K cache", atol=5e-3, rtol=5e-3)
        assert_close(layer.v.float().cpu().numpy(), Vo, what + ": V cache", atol=5e-3, rtol=5e-3)


def test_random_matmul_shapes_against_the_oracle(rx):
    """Seeded random (m, k, n) through relax_dequant_matmul (without and with the split-K workspace) and
    relax_half_matmul: any k that is a multiple of 8, any m, row counts on both sides of every dispatch boundary."""
    from test_gpu_parity import gpu_matmul, gpu_half_matmul
    rng = np.random.default_rng(77)
    for it in range(60):
        kind = it % 3
        n = int(rng.choice([1, 2, 3, 7, 16, 33, 64, 65, 100, 128, 129, 200, 300, 512, 513, 700]))
        if rng.random() < 0.4:
            n = int(rng.integers(1, 700))
        k = 8 * int(rng.integers(1, 1500)) if rng.random() < 0.5 else int(rng.choice([64, 128, 256, 1024, 2048, 4096, 8192, 11008]))
        m = int(rng.integers(1, 6000)) if rng.random() < 0.6 else int(rng.choice([64, 128, 256, 4096, 12288, 22016]))
        while m * k * n > 2e9:                              # keeps the oracle's share of the test to seconds
            if n > 16:
                n //= 2
            else:
                m //= 2
        what = "case %d (%s) m=%d k=%d n=%d" % (it, ["int4", "int4 + workspace", "fp16"][kind], m, k, n)
        x = wl.normal_f16_bits(400 + it, 1, (n, k))
        if kind < 2:
            q, s = wl.qmat(400 + it, 2, m, k)
            ref = oracle.dequant_matmul(wl.f16_bits_to_f32(x), q, s, m, k)
            got = gpu_matmul(rx, x, q, s, m, k, with_ws=bool(kind)).view(np.float16).astype(np.float32)
        else:
            w = (wl.f16_bits_to_f32(wl.normal_f16_bits(400 + it, 3, (m, k))) * 0.02).astype(np.float16).view(np.uint16)
            ref = oracle.half_matmul(wl.f16_bits_to_f32(x), w)
            got = gpu_half_matmul(rx, x, w)
        assert_close(got, ref, what)
        assert np.abs(got - ref).max() <= 2e-3 * max(1.0, np.abs(ref).max()), what


def test_random_attention_calls_against_the_oracle(rx):
    """Seeded random head layouts (1 to 8 KV heads, 1 to 8 query heads each, head dim 64 or 128), capacities, batch sizes
    and length mixes through relax_attention: decode batches, ragged prefills with and without a cached prefix, mixtures.
    The cache above every sequence's length holds NaNs, so a read past a row's position shows."""
    from test_gpu_parity import run_attention
    rng = np.random.default_rng(78)
    for it in range(45):
        d, g, group = int(rng.choice([64, 128])), int(rng.integers(1, 9)), int(rng.choice([1, 2, 4, 8]))
        cap, B = int(rng.choice([64, 130, 600, 1500])), int(rng.integers(1, 21))
        if it % 3 == 0:
            q = [1] * B
        elif it % 3 == 1:
            q = [int(rng.integers(1, min(cap, 200) + 1)) for _ in range(B)]
        else:
            q = [int(rng.choice([1, 1, int(rng.integers(2, min(cap, 50) + 1))])) for _ in range(B)]
        while sum(q) > 800:
            q[int(np.argmax(q))] //= 2
        q = [max(1, v) for v in q]
        kv = list(q) if it % 5 == 0 else [int(rng.integers(v, cap + 1)) for v in q]
        slots = [int(v) for v in rng.permutation(B + 3)[:B]]
        what = "case %d h=%d g=%d d=%d cap=%d q=%s kv=%s slots=%s" % (it, g * group, g, d, cap, q, kv, slots)
        got, ref = run_attention(rx, g * group, g, d, cap, B + 3, q, kv, slots, seed=600 + it)
        assert_close(got, ref, what, atol=2e-3, rtol=1e-2)
