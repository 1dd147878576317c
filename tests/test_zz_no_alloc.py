"""relax_attention_static -- the entry point that allocates nothing (its split-L partials live in a device array of the
library image) -- against relax_attention with a caller workspace: same kernels, so the outputs must be equal bit for
bit; and against the CPU oracle within the attention tolerance.  Two calls in a row share the array, the second on a
smaller input."""
import numpy as np
import pytest

import oracle
import workloads as wl
from helpers import assert_close, f32_cache

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def rx():
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    from paper_2311_02103_amd import binding
    binding.lib()
    return binding


def dev(a):
    from paper_2311_02103_amd.runtime import to_device
    return to_device(a)


def host_bits(t):
    from paper_2311_02103_amd.runtime import f16_bits
    return f16_bits(t)


def both_ways(rx, h, g, d, cap, slots, q_lens, kv_lens, slot_ids, seed):
    n = int(np.sum(q_lens))
    dims = rx.make_dims(h * d, h, g, d, 64, cap, slots)
    od = oracle.Dims(h * d, h, g, d, 64, kv_capacity=cap)
    kb, vb = (wl.normal_f16_bits(seed, 10 + j, (slots, cap, g, d)) for j in (0, 1))
    qb = wl.normal_f16_bits(seed, 12, (n, h, d))
    kc, vc = dev(kb), dev(vb)
    cache, seqs = rx.KVCache(kc, vc, None), rx.Seqs(q_lens, kv_lens, slot_ids)
    ws_bytes = rx.relax_workspace_bytes(dims, n, int(max(kv_lens)), len(q_lens))
    ws = torch.full((ws_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    want = torch.empty((n, h, d), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_attention(dev(qb), cache, seqs, dims, want, n, ws, ws_bytes), "relax_attention")
    got = torch.full((n, h, d), float("nan"), dtype=torch.float16, device="cuda")
    rx.check(rx.relax_attention_static(dev(qb), cache, seqs, dims, got, n), "relax_attention_static")
    torch.cuda.synchronize()
    ref = oracle.attention(wl.f16_bits_to_f32(qb), f32_cache(kb), f32_cache(vb), od, oracle.Seqs(q_lens, kv_lens, slot_ids))
    return host_bits(got), host_bits(want), ref


def test_static_attention_two_calls_second_smaller(rx):
    assert rx.relax_attention_static_max_bytes() == 16 << 20
    # first call: split-L decode of three sequences over long caches (many partials per row)
    got, want, ref = both_ways(rx, 32, 32, 128, 4096, 3, [1, 1, 1], [4096, 2500, 700], [2, 0, 1], seed=71)
    assert np.array_equal(got, want)
    assert_close(got.view(np.float16).astype(np.float32), ref, "static attention, long decode", atol=2e-3, rtol=1e-2)
    # second call, smaller: one short sequence; the array still holds the first call's partials
    got, want, ref = both_ways(rx, 32, 32, 128, 4096, 3, [1], [130], [1], seed=72)
    assert np.array_equal(got, want)
    assert_close(got.view(np.float16).astype(np.float32), ref, "static attention, short decode", atol=2e-3, rtol=1e-2)
    # grouped heads and a ragged mix of prefill and decode rows through the same array
    got, want, ref = both_ways(rx, 8, 2, 64, 300, 4, [5, 1, 37, 2], [9, 300, 37, 66], [3, 1, 0, 2], seed=73)
    assert np.array_equal(got, want)
    assert_close(got.view(np.float16).astype(np.float32), ref, "static attention, ragged", atol=2e-3, rtol=1e-2)
