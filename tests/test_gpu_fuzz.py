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
