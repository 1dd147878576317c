"""GPU tests of the device-resident descriptor (the runtime shape heap of Sec. 4.7 of the paper) and of graph offloading
(Sec. 4.5): a call whose kernels read positions from a device table gives the same bits as the call with host values,
and ONE captured decode step, replayed, walks through the positions like the eager loop does."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    from paper_2311_02103_amd import binding
    binding.lib()
    return binding


def table(q_lens, kv_lens, slots):
    """int32 [4][B] on the device: q_start, q_len, kv_len, slot."""
    starts = np.concatenate([[0], np.cumsum(q_lens)[:-1]])
    return torch.from_numpy(np.stack([starts, q_lens, kv_lens, slots]).astype(np.int32)).cuda().contiguous()


def bits(t):
    return t.view(torch.int16) if t.dtype == torch.float16 else t


@pytest.mark.parametrize("L", [1, 63, 300, 449, 2231, 4096])
def test_single_row_layer_reads_its_position_from_the_device_table(rx, L):
    """7B layer shape, one decode row: the folded attention path plans its splits on the device from the L it reads; the
    host only passes the capacity as the bound.  Output and appended cache rows equal the host-descriptor call bit for bit."""
    from paper_2311_02103_amd.runtime import DeviceLayer
    shape, cap = wl.LLAMA7B, 4096
    layer = DeviceLayer(wl.layer_weights(shape, 31), hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                        head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap, kv_slots=1, n_max=1, B_max=1)
    kb, vb = wl.kv_prefill(shape, 31, 1, cap)
    x = torch.from_numpy(wl.activations(shape, 31, L, 1).view(np.int16)).view(torch.float16).cuda()
    res = []
    for dev in (False, True):
        layer.load_cache(kb, vb)
        if dev:
            out = layer.forward(x, [1], [cap], None, device_table=table([1], [L], [0]))
        else:
            out = layer.forward(x, [1], [L], None)
        torch.cuda.synchronize()
        res.append((out.clone(), layer.k[0, L - 1].clone(), layer.v[0, L - 1].clone()))
    for name, a, b in zip(("out", "K row", "V row"), res[0], res[1]):
        assert torch.equal(bits(a), bits(b)), "%s differs at L=%d" % (name, L)
    assert torch.isfinite(res[0][0].float()).all() and float(res[0][0].float().abs().max()) > 0


def test_batched_decode_and_ragged_prefill_with_device_table(rx):
    """Few-row path (5 decode rows) and a ragged prefill (3 sequences, MFMA attention for the long one) with the
    descriptor on the device and loose host bounds: same bits as with host values."""
    from paper_2311_02103_amd.runtime import DeviceLayer
    shape, cap, B = wl.LLAMA7B, 256, 5
    layer = DeviceLayer(wl.layer_weights(shape, 32), hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                        head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap, kv_slots=B, n_max=64, B_max=B)
    kb, vb = wl.kv_prefill(shape, 32, B, cap)
    cases = [([1] * B, [7, 120, 64, 1, 200], [4, 3, 2, 1, 0]), ([20, 1, 9], [20, 77, 30], [2, 0, 1])]
    for q, kv, sl in cases:
        n = sum(q)
        x = torch.from_numpy(wl.activations(shape, 33, n, n).view(np.int16)).view(torch.float16).cuda()
        outs = []
        for dev in (False, True):
            layer.load_cache(kb, vb)
            if dev:
                out = layer.forward(x, q, [cap] * len(q), None, device_table=table(q, kv, sl))
            else:
                out = layer.forward(x, q, kv, sl)
            torch.cuda.synchronize()
            outs.append((out.clone(), layer.k.clone(), layer.v.clone()))
        for name, a, b in zip(("out", "K cache", "V cache"), outs[0], outs[1]):
            assert torch.equal(bits(a), bits(b)), "%s differs for q_lens %s" % (name, q)


def test_one_captured_decode_step_replays_through_the_positions(rx):
    """Graph offloading: the decode step of a 3-layer 7B-shaped model is captured ONCE (a one-element add that advances
    kv_len in the device table, then relax_model_step reading ids from the buffer it writes next_ids to) and replayed;
    every replay must give the logits and the token of the eager step with host values at that position.  Eager work
    and synchronisations sit between the replays."""
    from paper_2311_02103_amd.runtime import DeviceModel
    shape, V, nl, cap, P, steps = wl.LLAMA7B, 3000, 3, 96, 9, 6
    host = [wl.layer_weights(shape, 34, layer=l) for l in range(2)]
    mt = wl.model_tensors(shape, 34, V)
    dev = DeviceModel([host[l % 2] for l in range(nl)], mt["embedding"], mt["norm_final"], mt["lm_head"], hidden=shape.hidden,
                      n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap,
                      kv_slots=1, n_max=16, B_max=1)
    prompt = torch.from_numpy(wl.token_ids(34, P, V)).cuda()

    def prefill():
        for l in range(nl):
            dev.k[l].zero_()
            dev.v[l].zero_()
        _, nxt = dev.step(prompt, [P], [P])
        return nxt.clone()

    # eager loop with host values
    nxt = prefill()
    eager = []
    for s in range(steps):
        lg, nx = dev.step(nxt, [1], [P + 1 + s])
        torch.cuda.synchronize()
        eager.append((lg.clone(), nx.clone()))
        nxt = nx.clone()

    # one captured step, replayed
    ids = prefill()
    logits = torch.empty((1, V), dtype=torch.float16, device="cuda")
    tab = table([1], [P], [0])                                # kv_len is advanced inside the graph, before the step
    one = torch.ones((), dtype=torch.int32, device="cuda")
    stream = torch.cuda.Stream()

    def body():
        tab[2].add_(one)
        dev.step(ids, [1], [cap], logits=logits, next_ids=ids, stream=stream, device_table=tab)

    snap_k = [k.clone() for k in dev.k]
    snap_v = [v.clone() for v in dev.v]
    ids0 = ids.clone()
    with torch.cuda.stream(stream):
        body()                                                # everything touched once before capture
    stream.synchronize()
    for l in range(nl):                                       # undo the warm-up step
        dev.k[l].copy_(snap_k[l])
        dev.v[l].copy_(snap_v[l])
    ids.copy_(ids0)
    tab[2].fill_(P)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        body()
    for l in range(nl):                                       # capture does not run the work, but keep the state explicit
        dev.k[l].copy_(snap_k[l])
        dev.v[l].copy_(snap_v[l])
    ids.copy_(ids0)
    tab[2].fill_(P)
    torch.cuda.synchronize()
    for s in range(steps):
        with torch.cuda.stream(stream):
            graph.replay()
        stream.synchronize()
        scratch = torch.randn(1024, device="cuda").sum().item()      # eager work between the replays
        assert np.isfinite(scratch)
        assert int(tab[2].item()) == P + 1 + s
        assert torch.equal(bits(logits), bits(eager[s][0])), "logits of replay %d" % s
        assert torch.equal(ids, eager[s][1]), "token of replay %d" % s


def test_capture_of_a_call_with_more_than_sixteen_sequences_and_host_descriptors(rx):
    """21 sequences with host arrays: the descriptor does not fit kernel arguments, so the call writes a device table at the
    front of the workspace -- with small kernels that carry the values, no copy and no synchronisation, hence capturable.
    The captured call, replayed three times with eager work in between, gives the bits of the eager call every time."""
    from paper_2311_02103_amd.runtime import DeviceLayer
    shape, cap, B = wl.TINY, 64, 21
    layer = DeviceLayer(wl.layer_weights(shape, 41), hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                        head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap, kv_slots=B, n_max=B, B_max=B)
    kb, vb = wl.kv_prefill(shape, 41, B, cap)
    kv = [int(v) for v in wl.uniform_lengths(41, B, 2, 60)]
    slots = list(reversed(range(B)))
    x = torch.from_numpy(wl.activations(shape, 41, 0, B).view(np.int16)).view(torch.float16).cuda()
    layer.load_cache(kb, vb)
    want = layer.forward(x, [1] * B, kv, slots).clone()
    want_k = layer.k.clone()
    torch.cuda.synchronize()

    stream = torch.cuda.Stream()
    out = torch.empty_like(x)
    call = layer.prepare(x, [1] * B, kv, slots, out=out)
    layer.load_cache(kb, vb)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        call(stream.cuda_stream)
    for rep in range(3):
        layer.load_cache(kb, vb)                       # eager work between the replays; the appended rows are written again
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(bits(out), bits(want)), "replay %d: output differs from the eager call" % rep
        assert torch.equal(bits(layer.k), bits(want_k)), "replay %d: K cache differs" % rep


MID = wl.LayerShape("table-mid", hidden=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn=5632)


def half_weights(shape, seed):
    w = {}
    for j, (name, (m, k)) in enumerate(shape.matrices().items()):
        w[name] = (wl.normal_f32(seed, 40 + j, (m, k)) * np.float32(0.02)).astype(np.float16).view(np.uint16)
    for j, name in enumerate(("norm_attn", "norm_ffn")):
        w[name] = wl.normal_f16_bits(seed, 50 + j, (shape.hidden,), std=0.1, mean=1.0)
    return w


@pytest.mark.parametrize("kind", ["q3", "f16"])
@pytest.mark.parametrize("L", [1, 63, 300, 512])
def test_single_row_of_the_3bit_and_fp16_layers_reads_its_position_from_the_device_table(rx, kind, L):
    """The fused one-row path of the layers on 3-bit and on fp16 weights: with the device table the kernels read the position
    and plan the attention splits on the device; output and appended cache rows equal the host-descriptor call bit for bit."""
    from paper_2311_02103_amd.runtime import DeviceLayerF16, DeviceLayerQ3
    shape, cap = MID, 512
    kw = dict(hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn,
              kv_capacity=cap, kv_slots=1, n_max=1, B_max=1)
    layer = DeviceLayerQ3(wl.layer_weights3(shape, 37), **kw) if kind == "q3" else DeviceLayerF16(half_weights(shape, 37), **kw)
    kb, vb = wl.kv_prefill(shape, 37, 1, cap)
    x = torch.from_numpy(wl.activations(shape, 37, L, 1).view(np.int16)).view(torch.float16).cuda()
    res = []
    for dev in (False, True):
        layer.load_cache(kb, vb)
        if dev:
            out = layer.forward(x, [1], [cap], None, device_table=table([1], [L], [0]))
        else:
            out = layer.forward(x, [1], [L], None)
        torch.cuda.synchronize()
        res.append((out.clone(), layer.k[0, L - 1].clone(), layer.v[0, L - 1].clone()))
    for name, a, b in zip(("out", "K row", "V row"), res[0], res[1]):
        assert torch.equal(bits(a), bits(b)), "%s differs at L=%d (%s)" % (name, L, kind)
    assert torch.isfinite(res[0][0].float()).all() and float(res[0][0].float().abs().max()) > 0


@pytest.mark.parametrize("L", [1, 300, 512])
def test_single_row_layer_at_hidden_5120_reads_its_position_from_the_device_table(rx, L):
    """Hidden width of the 13B shape (three chunks of 2048 columns, the attention merge folded into a three-chunk output
    projection): device-table call and host-descriptor call give the same bits."""
    from paper_2311_02103_amd.runtime import DeviceLayer
    shape, cap = wl.LayerShape("h5120", hidden=5120, n_heads=40, n_kv_heads=40, head_dim=128, ffn=1024), 512
    layer = DeviceLayer(wl.layer_weights(shape, 41), hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                        head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap, kv_slots=1, n_max=1, B_max=1)
    kb, vb = wl.kv_prefill(shape, 41, 1, cap)
    x = torch.from_numpy(wl.activations(shape, 41, L, 1).view(np.int16)).view(torch.float16).cuda()
    res = []
    for dev in (False, True):
        layer.load_cache(kb, vb)
        if dev:
            out = layer.forward(x, [1], [cap], None, device_table=table([1], [L], [0]))
        else:
            out = layer.forward(x, [1], [L], None)
        torch.cuda.synchronize()
        res.append((out.clone(), layer.k[0, L - 1].clone(), layer.v[0, L - 1].clone()))
    for name, a, b in zip(("out", "K row", "V row"), res[0], res[1]):
        assert torch.equal(bits(a), bits(b)), "%s differs at L=%d" % (name, L)
    assert torch.isfinite(res[0][0].float()).all() and float(res[0][0].float().abs().max()) > 0
