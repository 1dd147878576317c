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
             ([241, 199, 128], [241, 2048, 128], [3, 1, 2])]                   # tiled GEMM, fresh prefills and a full cache
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
