"""GPU parity of relax_model_step (embedding, layer stack, final norm, fp16 LM head, greedy pick) against the oracle's
model_step, teacher-forced: both sides are always fed the oracle's token stream, logits are compared per step under
the fp16 tolerance, and a greedy pick may only differ where the oracle's top two logits are closer than the tolerance
allows to separate."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from helpers import assert_close, oracle_dims, oracle_weights, f32_cache

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rx():
    from paper_2311_02103_amd import binding
    binding.lib()
    return binding


def build_models(shape, n_layers, vocab, seed, cap, slots, n_max, B_max, distinct_layers=None):
    """The same host arrays as an oracle model (dims, layers, tensors) and a DeviceModel.  Layers cycle through
    `distinct_layers` weight sets (all distinct by default)."""
    from paper_2311_02103_amd.runtime import DeviceModel
    distinct = distinct_layers or n_layers
    host = [wl.layer_weights(shape, seed, layer=l) for l in range(min(distinct, n_layers))]
    per_layer = [host[l % len(host)] for l in range(n_layers)]
    mt = wl.model_tensors(shape, seed, vocab)
    dev = DeviceModel(per_layer, mt["embedding"], mt["norm_final"], mt["lm_head"], hidden=shape.hidden, n_heads=shape.n_heads,
                      n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap, kv_slots=slots,
                      n_max=n_max, B_max=B_max, rms_eps=shape.rms_eps, rope_base=shape.rope_base)
    od = oracle_dims(shape, cap)
    ol = [oracle_weights(shape, w) for w in per_layer]
    return dev, od, ol, mt


def check_step(dev, od, ol, mt, ids, q_lens, kv_lens, slots, Ko, Vo, what):
    """One teacher-forced step on both sides; returns the oracle's greedy ids."""
    logits, nxt = dev.step(torch.from_numpy(np.asarray(ids, np.int32)).cuda(), q_lens, kv_lens, slots)
    torch.cuda.synchronize()
    ref_logits, ref_ids = oracle.model_step(od, ol, mt["embedding"], mt["norm_final"], mt["lm_head"], np.asarray(ids, np.int32), Ko, Vo,
                                            oracle.Seqs(q_lens, kv_lens, slots))
    got = logits.float().cpu().numpy()
    # A logit is a sum over `hidden` terms of fp16-rounded activations, so its absolute error grows with the scale of
    # the logits themselves: the absolute part of the tolerance is taken relative to their RMS once that exceeds 1
    # (70B shape: hidden 8192, logits of RMS 1.8; 512 000 values per step, i.e. a five-sigma tail).
    atol = 1e-2 * max(1.0, float(np.sqrt(np.mean(np.square(ref_logits)))))
    assert_close(got, ref_logits, what + " logits", atol=atol)
    got_ids = nxt.cpu().numpy()
    # the library picks from the fp16 logits it stores: its pick must be a maximum of them (lowest index among ties) ...
    for b in range(len(q_lens)):
        assert got_ids[b] == int(np.argmax(got[b])), what + ": pick is not the first maximum of the stored logits"
        # ... and may differ from the oracle's only inside the tolerance band around the oracle's top value
        if got_ids[b] != ref_ids[b]:
            top = ref_logits[b, ref_ids[b]]
            assert top - ref_logits[b, got_ids[b]] <= 2 * (atol + 2e-2 * abs(top)), what + ": greedy pick outside the tolerance band"
    return ref_ids


def zero_caches(od, n_layers, slots):
    shp = (slots, od.kv_capacity, od.n_kv_heads, od.head_dim)
    return [np.zeros(shp, np.float32) for _ in range(n_layers)], [np.zeros(shp, np.float32) for _ in range(n_layers)]


@pytest.mark.parametrize("B", [1, 3, 8, 11, 16])
def test_embedding_norm_head_argmax_without_layers(rx, B):
    """n_layers = 0 isolates gather -> final norm -> LM head (passes of 8, 2, 1 rows) -> greedy pick; vocab 1003 is ragged."""
    dev, od, ol, mt = build_models(wl.TINY, 0, 1003, seed=11, cap=8, slots=B, n_max=B, B_max=B)
    ids = wl.token_ids(11, B, 1003)
    check_step(dev, od, ol, mt, ids, [1] * B, [1] * B, None, [], [], "head-only B=%d" % B)


def test_head_uses_last_row_of_each_sequence(rx):
    dev, od, ol, mt = build_models(wl.TINY, 0, 500, seed=12, cap=16, slots=3, n_max=12, B_max=3)
    ids = wl.token_ids(12, 12, 500)
    check_step(dev, od, ol, mt, ids, [5, 1, 6], [5, 9, 6], [2, 0, 1], [], [], "ragged head-only")


def test_out_of_range_token_raises_the_flag(rx):
    dev, od, ol, mt = build_models(wl.TINY, 0, 100, seed=13, cap=8, slots=2, n_max=2, B_max=2)
    assert rx.relax_workspace_error(dev.dims, dev.ws) == 0
    dev.step(torch.tensor([5, 100], dtype=torch.int32).cuda(), [1, 1], [1, 1])
    torch.cuda.synchronize()
    assert rx.relax_workspace_error(dev.dims, dev.ws) & 2


def test_tiny_model_prefill_then_teacher_forced_decode(rx):
    """Schedule of the small configuration on a 3-layer stack: one 37-row prefill, then 16 decode steps."""
    V, nl = 2000, 3
    dev, od, ol, mt = build_models(wl.TINY, nl, V, seed=14, cap=64, slots=1, n_max=37, B_max=1)
    Ko, Vo = zero_caches(od, nl, 1)
    prompt = wl.token_ids(14, 37, V)
    nxt = check_step(dev, od, ol, mt, prompt, [37], [37], None, Ko, Vo, "prefill 37")
    for step in range(16):
        L = 38 + step
        nxt = check_step(dev, od, ol, mt, nxt, [1], [L], None, Ko, Vo, "decode L=%d" % L)
    # the device caches hold what the oracle's hold (fp16 rounding apart)
    for l in range(nl):
        assert_close(dev.k[l].float().cpu().numpy()[0, :53], Ko[l][0, :53], "K cache layer %d" % l, atol=4e-3, rtol=4e-3)


def test_tiny_model_ragged_batch_with_many_sequences(rx):
    V, nl, B = 700, 2, 19                                  # more sequences than ride in kernel arguments
    dev, od, ol, mt = build_models(wl.TINY, nl, V, seed=15, cap=48, slots=B, n_max=64, B_max=B)
    Ko, Vo = zero_caches(od, nl, B)
    q = [int(v) for v in wl.uniform_lengths(15, B, 1, 5)]
    ids = wl.token_ids(15, sum(q), V)
    nxt = check_step(dev, od, ol, mt, ids, q, q, list(range(B)), Ko, Vo, "ragged prefill")
    kv = [a + 1 for a in q]
    check_step(dev, od, ol, mt, nxt, [1] * B, kv, list(range(B)), Ko, Vo, "batched decode")


def test_7b_shape_two_layers_prefill_and_decode(rx):
    """7B layer shape, vocab 32000, two layers: a 24-row prefill (MFMA path) and three teacher-forced decode steps."""
    shape, V, nl = wl.LLAMA7B, 32000, 2
    dev, od, ol, mt = build_models(shape, nl, V, seed=16, cap=64, slots=1, n_max=24, B_max=1, distinct_layers=1)
    Ko, Vo = zero_caches(od, nl, 1)
    nxt = check_step(dev, od, ol, mt, wl.token_ids(16, 24, V), [24], [24], None, Ko, Vo, "7B prefill 24")
    for step in range(3):
        nxt = check_step(dev, od, ol, mt, nxt, [1], [25 + step], None, Ko, Vo, "7B decode %d" % step)


def test_70b_shape_batched_decode_one_layer(rx):
    """Batched-decode configuration at the 70B layer shape (GQA 64/8, hidden 8192), B = 16, L_b ~ U{100..8000}, one layer
    + head: layer-local parity for the big configuration (the full 80-layer stack is the same call 80 times)."""
    shape, V, B, cap = wl.LLAMA70B, 32000, 16, 8192
    dev, od, ol, mt = build_models(shape, 1, V, seed=17, cap=cap, slots=B, n_max=B, B_max=B)
    kv = [int(v) for v in wl.uniform_lengths(17, B, 100, 8000)]
    kb, vb = wl.kv_prefill(shape, 17, B, cap)
    dev.k[0].copy_(torch.from_numpy(kb.view(np.int16)).view(torch.float16).cuda())
    dev.v[0].copy_(torch.from_numpy(vb.view(np.int16)).view(torch.float16).cuda())
    Ko, Vo = [f32_cache(kb)], [f32_cache(vb)]
    check_step(dev, od, ol, mt, wl.token_ids(17, B, V), [1] * B, kv, list(range(B)), Ko, Vo, "70B-shape batched decode")


@pytest.mark.parametrize("q", [None, [150, 50]])
def test_few_row_path_with_and_without_folded_finishing_steps(rx, q):
    """The few-row matrix path folds rotary + append and the RMSNorms into the finishing pass of its split-K matmuls
    (and the first RMSNorm of a layer into the last finishing pass of the layer before).  The folded kernels repeat the
    arithmetic of the separate ones element by element, so logits, picks and caches must be identical bit for bit."""
    shape, V, nl = wl.LLAMA7B, 3000, 3
    if q is None:                                          # five short prompts: every matmul is the few-row kernel
        B, cap = 5, 64
        q = [int(v) for v in wl.uniform_lengths(21, B, 1, 6)]
    else:                                                  # 200 rows: the tiled GEMM, cut along k for the output and down projections
        B, cap = len(q), 256
    dev, od, ol, mt = build_models(shape, nl, V, seed=21, cap=cap, slots=B, n_max=max(32, sum(q)), B_max=B, distinct_layers=2)
    ids = torch.from_numpy(wl.token_ids(21, sum(q), V)).cuda()
    results = []
    try:
        for folded in (0, 1):
            rx.check(rx.relax_set_option("fuse_finish", folded))
            for l in range(nl):
                dev.k[l].zero_()
                dev.v[l].zero_()
            lg1, nx1 = dev.step(ids, q, q, list(range(B)))
            lg1, nx1 = lg1.clone(), nx1.clone()
            lg2, nx2 = dev.step(nx1, [1] * B, [a + 1 for a in q], list(range(B)))
            torch.cuda.synchronize()
            results.append((lg1.cpu(), nx1.cpu(), lg2.clone().cpu(), nx2.clone().cpu(), [k.clone().cpu() for k in dev.k], [v.clone().cpu() for v in dev.v]))
    finally:
        rx.check(rx.relax_set_option("fuse_finish", 1))      # back to the default
    a, b = results
    for name, x, y in (("prefill logits", a[0], b[0]), ("prefill picks", a[1], b[1]), ("decode logits", a[2], b[2]), ("decode picks", a[3], b[3])):
        assert torch.equal(x.view(torch.int16) if x.dtype == torch.float16 else x, y.view(torch.int16) if y.dtype == torch.float16 else y), name
    for l in range(nl):
        assert torch.equal(a[4][l].view(torch.int16), b[4][l].view(torch.int16)), "K cache layer %d" % l
        assert torch.equal(a[5][l].view(torch.int16), b[5][l].view(torch.int16)), "V cache layer %d" % l
    assert float(a[0].float().abs().max()) > 0 and torch.isfinite(a[2].float()).all()


SCHEDULE_SHAPES = [(wl.TINY, 1003, 3, 12, 96),
                   (wl.LayerShape("mid-gqa", hidden=1024, n_heads=16, n_kv_heads=4, head_dim=64, ffn=2816), 5000, 2, 8, 300),
                   (wl.LayerShape("mid-mha", hidden=2048, n_heads=16, n_kv_heads=16, head_dim=128, ffn=5632), 32000, 2, 20, 160)]


@pytest.mark.parametrize("si", range(len(SCHEDULE_SHAPES)))
def test_serving_like_schedule_against_the_oracle(rx, si):
    """A seeded continuous-batching schedule through relax_model_step: every step retires some sequences, admits new
    prompts into free cache slots and decodes the rest, in shuffled order, so calls mix prefill and decode rows, the
    slots in use and the batch size change from call to call, and each sequence's cache is what earlier calls left."""
    shape, V, nl, slots, cap = SCHEDULE_SHAPES[si]
    n_max = 400
    rng = np.random.default_rng(900 + si)
    dev, od, ol, mt = build_models(shape, nl, V, seed=90 + si, cap=cap, slots=slots, n_max=n_max, B_max=slots)
    Ko, Vo = zero_caches(od, nl, slots)
    length, last = {}, {}                                  # per live slot: cached length, the oracle's last pick
    for step in range(12):
        for s in list(length):
            if length[s] + 1 >= cap or rng.random() < 0.15:
                del length[s], last[s]
        free = [s for s in range(slots) if s not in length]
        rng.shuffle(free)
        admit = free[:int(rng.integers(0, min(len(free), 4) + 1))]
        if not length and not admit:
            admit = free[:1]
        order = list(length) + admit
        rng.shuffle(order)
        sl, q, kv, ids = [], [], [], []
        for s in order:
            sl.append(s)
            if s in length:
                q.append(1), kv.append(length[s] + 1), ids.append([last[s]])
            else:
                p = int(rng.integers(1, min(cap - 2, 70)))
                q.append(p), kv.append(p), ids.append(list(wl.token_ids(1000 * si + step, p, V)))
        while sum(q) > n_max:
            j = int(np.argmax(q))
            q[j] //= 2
            kv[j], ids[j] = q[j], ids[j][:q[j]]
        flat = np.asarray([t for row in ids for t in row], np.int32)
        nxt = check_step(dev, od, ol, mt, flat, q, kv, sl, Ko, Vo, "%s step %d q=%s kv=%s slots=%s" % (shape.name, step, q, kv, sl))
        for b, s in enumerate(sl):
            length[s], last[s] = kv[b], int(nxt[b])
