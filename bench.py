#!/usr/bin/env python3
"""Benchmarks of the decoder-layer hot path on one MI355X.  Prints ONE JSON line per run.

Default workload (configs[1] of the benchmark spec, the one the headline metric is quoted on):
  decode_layer   one Llama-2-7B-shaped int4 (group 32) decoder layer, batch 1, n = 1, KV length L drawn uniformly
                 from 1..4096 for each of 64 seeded calls, fp16 KV cache pre-filled with N(0,1).  A step is one call of
                 relax_decoder_layer = one token through one layer.  Consecutive steps use different weight sets
                 (8 sets, 911 MB) so the 256 MB last-level cache cannot hold the weights: the int4 stream comes from HBM.
Other workloads (--workload), same JSON schema, for the other configurations:
  prefill_layer  configs[2]: the same layer on n rows (default 2048), L = n, empty cache; a step is one call.
  model_7b       configs[3]: 32 layers + fp16 embedding / LM head, 128-token prompt, then greedy decode at batch 1;
                 a step is one relax_model_step call = one generated token.
  batched_70b    configs[4]: Llama-2-70B-shaped GQA model, 80 layers, 16 sequences with L_b ~ U{100..8000};
                 a step is one relax_model_step call = 16 generated tokens.
  ceilings       what this device reaches on a plain streaming read, a chain of streaming launches and a bare MFMA loop.
  batch_sweep    one 7B-shaped layer call on n decode rows against n (where the dispatch on n changes kernels).
  memory_plan    host-only: planned against unplanned bytes of the layer's intermediates (Alg. 3 of the paper).
  half_sweep     relax_half_matmul (plain fp16 weights) against n, matvec passes and tiled GEMM forced in turn: the crossover.
  decode_shapes  one decode row (L = 2231) through one int4 layer of the 7B, 13B and 70B shapes: the same binary on three sizes.
  q3_matvec      relax_dequant_matmul_q3_native / relax_dequant_matmul_q3 (3-bit weights) at n = 1 on the four matrix shapes of the 7B layer.
All inputs are seeded and synthetic and resident in HBM before the timed region.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0           # MI355X published HBM3E bandwidth
PEAK_MFMA_TFLOPS = 2500.0       # MI355X published dense fp16 MFMA rate
STEP_NAMES = ["qkv", "attention", "o_proj", "gate_up", "down"]


def traffic_from_profile(name):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, calibrated on a copy kernel),
    stored next to the profile summary it came from; None when that file is not there."""
    path = os.path.join(ROOT, "profiles", name)
    if os.path.exists(path):
        return json.load(open(path)).get("hbm_bytes_per_launch")
    return None


def time_steps(torch, rx, stream, call, step_ids, reps):
    """Average duration (ms) of single steps of the layer, HIP events on the launch stream through the ABI's hook."""
    import numpy as np
    out = {}
    for sid in step_ids:
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:                            # materialise the hipEvent handles
            a.record(stream), b.record(stream)
        stream.synchronize()
        for i, (a, b) in enumerate(evs):
            rx.relax_profile_step_events(a.cuda_event, b.cuda_event, sid)
            call(i)
        stream.synchronize()
        out[STEP_NAMES[sid]] = float(np.mean([a.elapsed_time(b) for a, b in evs]))
    return out


def emit(args, metric, unit, value, ms_per_step, dtype, config, roofline, cpu, extra):
    line = {"metric": metric, "value": round(value, 1), "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": dtype, "data": "synthetic", "config": config}
    line.update(extra)
    line["roofline"] = roofline
    line["cpu_baseline"] = cpu
    print(json.dumps(line))


# ------------------------------------------------------------------------------------------------ the other two parts of the metric
def measure_prefill(np, torch, wl, rx, host_w, n=2048, calls=30):
    """configs[2] at n rows, short: ms per layer call and the MFMA rate of its GEMMs (HIP events around each step)."""
    from paper_2311_02103_amd.runtime import DeviceLayer, to_device
    shape = wl.LLAMA7B
    layer = DeviceLayer(host_w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                        ffn=shape.ffn, kv_capacity=n, n_max=n)
    x = to_device(wl.activations(shape, 2, 0, n))
    out = torch.empty_like(x)
    stream = torch.cuda.Stream()
    call = layer.prepare(x, [n], [n], out=out)
    for _ in range(10):                      # as the prefill_layer workload: ten untimed calls first
        call(stream.cuda_stream)
    stream.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(calls):
        call(stream.cuda_stream)
    e1.record(stream)
    stream.synchronize()
    ms = e0.elapsed_time(e1) / calls
    kms = time_steps(torch, rx, stream, lambda i: call(stream.cuda_stream), [0, 1, 2, 3, 4], calls)
    P = sum(m * k for m, k in shape.matrices().values())
    m, k = shape.matrices()["wgu"]
    gemm_ms = kms["qkv"] + kms["o_proj"] + kms["gate_up"] + kms["down"]
    gu = 2.0 * n * m * k / kms["gate_up"] / 1e9
    allg = 2.0 * n * P / gemm_ms / 1e9
    return {"workload": "configs[2]: the same 7B-shaped layer, prefill of n=%d rows, L=n (same binary)" % n, "ms_per_call": round(ms, 4),
            "tokens_per_s": round(n / ms * 1e3, 1), "gate_up_gemm_TFLOPs": round(gu, 1), "gate_up_frac_of_mfma_peak": round(gu / PEAK_MFMA_TFLOPS, 4),
            "four_gemm_steps_TFLOPs": round(allg, 1), "frac_of_mfma_peak": round(allg / PEAK_MFMA_TFLOPS, 4),
            "attention_ms": round(kms["attention"], 4), "note": "the qkv step includes the RMSNorm and rotary/append launches"}


def measure_model_7b(np, torch, wl, rx, host_sets, steps=64):
    """configs[3], short: 32 layers (the weight sets cycled) + fp16 embedding and LM head, 128-token prompt, then greedy decode."""
    from paper_2311_02103_amd.runtime import DeviceModel
    shape, nl, V, cap, seed = wl.LLAMA7B, 32, 32000, 512, 3
    mt = wl.model_tensors(shape, seed, V)
    dev = DeviceModel([host_sets[l % len(host_sets)] for l in range(nl)], mt["embedding"], mt["norm_final"], mt["lm_head"], hidden=shape.hidden,
                      n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap,
                      kv_slots=1, n_max=128, B_max=1)
    logits = torch.empty((1, V), dtype=torch.float16, device="cuda")
    nxt = torch.empty((1,), dtype=torch.int32, device="cuda")
    dev.step(torch.from_numpy(wl.token_ids(seed, 128, V)).cuda(), [128], [128], logits=logits, next_ids=nxt)
    for s in range(8):
        dev.step(nxt, [1], [129 + s], logits=logits, next_ids=nxt)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(8, 8 + steps):
        dev.step(nxt, [1], [129 + s], logits=logits, next_ids=nxt)
    torch.cuda.synchronize()
    el = time.perf_counter() - t0
    P = sum(m * k for m, k in shape.matrices().values())
    step_bytes = nl * P * 0.5625 + V * shape.hidden * 2 + shape.kv_bytes_per_token() * (137 + steps / 2.0) * nl
    tps = steps / el
    return {"workload": "configs[3]: 32-layer 7B-shaped model (%d weight sets cycled), vocab 32000, 128-token prompt, then %d greedy decode "
                        "steps at batch 1, one C call per token" % (len(host_sets), steps),
            "tokens_per_s": round(tps, 1), "ms_per_token": round(el * 1e3 / steps, 4), "bytes_per_token": int(step_bytes),
            "achieved_GBps": round(step_bytes * tps / 1e9, 1), "frac_of_hbm_peak": round(step_bytes * tps / 1e9 / PEAK_HBM_GBS, 4),
            "hbm_ceiling_tokens_per_s": round(PEAK_HBM_GBS * 1e9 / step_bytes, 1)}


# ------------------------------------------------------------------------------------------------ configs[1]
def bench_decode_layer(args, np, torch, wl, rx):
    from paper_2311_02103_amd.runtime import DeviceLayer, f16_bits, to_device
    args.mode = args.mode or "graph"
    dev = "cuda:0"
    shape, cap, seed, ncalls = wl.LLAMA7B, 4096, 1, 64
    steps = args.steps = args.steps or 1280
    warmup = args.warmup = 128 if args.warmup is None else args.warmup

    t_setup = time.time()
    Ls = [int(v) for v in wl.uniform_lengths(seed, ncalls, 1, cap)]
    kv_k, kv_v = wl.kv_prefill(shape, seed, 1, cap)
    host_w0, layers, host_sets = None, [], []
    for s in range(args.sets):
        w = wl.layer_weights(shape, seed, layer=s)
        host_sets.append(w)
        if s == 0:
            host_w0 = w
        lay = DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                          ffn=shape.ffn, kv_capacity=cap, n_max=1, device=dev, share_from=layers[0] if layers else None)
        lay.load_cache(kv_k, kv_v)
        layers.append(lay)
    xs_host = [wl.activations(shape, seed, c, 1) for c in range(ncalls)]
    xs = [to_device(x, dev) for x in xs_host]
    outs = [torch.empty_like(x) for x in xs]
    calls = [layers[c % args.sets].prepare(xs[c], [1], [Ls[c]], out=outs[c]) for c in range(ncalls)]
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    stream = torch.cuda.Stream()
    sh = stream.cuda_stream

    def run_eager(nsteps, first=0):
        for i in range(first, first + nsteps):
            calls[i % ncalls](sh)

    # The timed region is `steps` consecutive calls of the 64-call schedule, repeated `reps` times so that it lasts at least
    # 0.2 s whatever --steps is (a handful of 45 us steps would time the clock, not the GPU); ms_per_step is the mean over all
    # of them.  Graph mode (Sec. 4.5 of the paper): the calls are captured once -- the whole schedule in one graph, what is
    # left of `steps` after whole schedules in a second one -- and replayed; eager mode issues one C call per step.
    def capture(first, count):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            run_eager(count, first)
        return g

    full, rest = divmod(steps, ncalls)
    graph = graph_rest = None
    if args.mode == "graph":
        with torch.cuda.stream(stream):
            run_eager(ncalls)                       # everything touched once before capture
        stream.synchronize()
        graph = capture(0, ncalls)
        graph_rest = capture(0, rest) if rest else None

    def run(nsteps):
        f, r = divmod(nsteps, ncalls)
        if graph is None:
            run_eager(nsteps)
            return
        with torch.cuda.stream(stream):
            for _ in range(f):
                graph.replay()
            if r == rest and graph_rest is not None:
                graph_rest.replay()
        if r != rest:
            run_eager(r)

    run(warmup)
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(steps)
    stream.synchronize()
    first_pass = time.perf_counter() - t0
    passes = max(1, min(10000, int(0.25 / max(first_pass, 1e-6)) + 1))
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(passes):
        run(steps)
    stream.synchronize()
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t0) / passes     # per pass of `steps` steps
    ms_per_step = elapsed * 1e3 / steps

    mean_L = float(np.mean([Ls[i % ncalls] for i in range(steps)]))
    kvb = shape.kv_bytes_per_token()
    layer_bytes = shape.packed_bytes_per_layer() + kvb * mean_L + kvb + 6 * shape.hidden * 2
    layer_gbs = layer_bytes / (ms_per_step * 1e-3) / 1e9

    kernel_ms, roofline = {}, None
    if not args.no_kernel_timing:
        ids = [0, 1, 2, 3, 4]
        kernel_ms = time_steps(torch, rx, stream, lambda i: calls[i % ncalls](sh), ids, min(steps, 256))
        if graph is not None:
            # The event pair around one eager launch also sees the gap before it.  Inside the captured schedule the
            # kernels run back to back, so the duration of the gate/up launch there is what one more launch of it per
            # call adds: the same schedule captured with that (idempotent) launch doubled, both timed with HIP events
            # on the launch stream over the same number of replays.
            # The extra launch reads the gate/up matrix of the weight set half a rotation away, which is as cold as the
            # real one (with the same matrix it would be served from the memory-side cache).
            graph2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph2, stream=stream):
                for c in range(ncalls):
                    other = layers[(c + args.sets // 2) % args.sets]
                    rx.relax_profile_alt_gate_up(other.t["wgu.q"], other.t["wgu.s"])
                    calls[c](sh)
            rx.relax_profile_alt_gate_up(None, None)
            reps = max(2, min(steps // ncalls, 20))

            def replay_ms(g):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                with torch.cuda.stream(stream):
                    g.replay()
                    e0.record(stream)
                    for _ in range(reps):
                        g.replay()
                    e1.record(stream)
                stream.synchronize()
                return e0.elapsed_time(e1) / (reps * ncalls)
            base = min(replay_ms(graph) for _ in range(3))
            doubled = min(replay_ms(graph2) for _ in range(3))
            kernel_ms["gate_up_eager_events"] = kernel_ms["gate_up"]
            kernel_ms["gate_up"] = doubled - base
            kernel_ms["step_in_graph_events"] = base
    m, k = shape.matrices()["wgu"]
    gu_bytes = m * (k // 2) + m * (k // 32) * 2 + shape.hidden * 4 + shape.hidden * 2 + shape.ffn * 2
    if "gate_up" in kernel_ms:
        ach = gu_bytes / (kernel_ms["gate_up"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "gemv_q4_reg_kernel<X_F32_NORM, EPI_SWIGLU, 2> (gate/up matvec, m=22016, k=4096: "
                                                "RMSNorm prologue, SwiGLU epilogue)",
                    "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4),
                    "traffic": traffic_from_profile("traffic_gate_up_matvec_7b.json"),
                    "traffic_source": "stored value, not measured in this run: profiles/traffic_gate_up_matvec_7b.json (rocprofv3 --pmc "
                                      "FETCH_SIZE and WRITE_SIZE of this kernel, scaled by a copy kernel of known size)",
                    "algorithmic_bytes_per_launch": gu_bytes, "avg_launch_ms": round(kernel_ms["gate_up"], 5)}

    # CPU baseline: the oracle as it stands on the calls of weight set 0, cycled until the time budget is used; the first
    # pass doubles as a parity check of the very calls that were timed.
    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        mats = shape.matrices()
        ow = oracle.LayerWeights(*(oracle.QMat(host_w0[nm + ".q"], host_w0[nm + ".s"], *mats[nm]) for nm in ("wqkv", "wo", "wgu", "wdown")),
                                 host_w0["norm_attn"], host_w0["norm_ffn"])
        od = oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.rms_eps, shape.rope_base, cap)
        Kf = wl.f16_bits_to_f32(kv_k).reshape(1, cap, shape.n_kv_heads, shape.head_dim)
        Vf = wl.f16_bits_to_f32(kv_v).reshape(1, cap, shape.n_kv_heads, shape.head_dim)
        sample = [c for c in range(ncalls) if c % args.sets == 0]
        layers[0].load_cache(kv_k, kv_v)            # both sides start from the seeded pre-fill and append in the same order
        torch.cuda.synchronize()
        done, t_cpu, worst, checked = 0, 0.0, 0.0, 0
        while t_cpu < args.cpu_seconds:
            for c in sample:
                t1 = time.perf_counter()
                ref = oracle.decoder_layer(od, ow, xs_host[c], Kf, Vf, oracle.Seqs([1], [Ls[c]]))
                t_cpu += time.perf_counter() - t1
                done += 1
                if checked < len(sample):
                    calls[c](sh)
                    stream.synchronize()
                    got = f16_bits(outs[c]).view(np.float16).astype(np.float32)
                    err = np.abs(got - ref)
                    assert np.all(err <= 1e-2 + 2e-2 * np.abs(ref)), "bench: GPU output of call %d is outside tolerance" % c
                    worst, checked = max(worst, float(err.max())), checked + 1
                if t_cpu >= args.cpu_seconds:
                    break
        cpu = {"value": round(done / t_cpu, 3), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%d layer calls (the %d calls of the schedule that use weight set 0, cycled), %.1f s of oracle time; GPU "
                         "outputs of those calls checked against it, max abs err %.2e" % (done, len(sample), t_cpu, worst)}

    # the other two parts of the benchmark's metric, from short runs in this process: prefill MFMA utilisation, model-level rate
    extra_parts = {}
    if not args.no_extras:
        del calls, xs, outs
        for lay in layers:
            lay.t.clear()
        layers.clear()
        torch.cuda.empty_cache()
        extra_parts["prefill"] = measure_prefill(np, torch, wl, rx, host_w0)
        torch.cuda.empty_cache()
        extra_parts["model_7b"] = measure_model_7b(np, torch, wl, rx, host_sets)

    emit(args, "decode tokens/s (7B-shaped int4, batch 1)", "tokens/s", steps / elapsed, ms_per_step,
         "f16 (int4 weights, f32 accumulate)",
         {"workload": "configs[1]: one Llama-2-7B-shaped int4-g32 decoder layer, decode only, batch 1, n=1, L~U{1..4096} over 64 "
                      "seeded calls; 1 step = 1 token through 1 layer (a 32-layer model does 32 such steps per token); %d rotating "
                      "weight sets" % args.sets,
          "mode": args.mode, "timed_passes": passes, "mean_L": round(mean_L, 1), "build_id": rx.relax_build_id(), "setup_s": round(setup_s, 1)},
         roofline, cpu,
         {"layer_hbm": {"algorithmic_bytes_per_step": int(layer_bytes), "achieved_GBps": round(layer_gbs, 1),
                        "frac_of_peak": round(layer_gbs / PEAK_HBM_GBS, 4)},
          "kernel_ms": {k_: round(v, 5) for k_, v in kernel_ms.items()}, **extra_parts})


# ------------------------------------------------------------------------------------------------ configs[2]
def bench_prefill_layer(args, np, torch, wl, rx):
    from paper_2311_02103_amd.runtime import DeviceLayer, f16_bits, to_device
    shape, seed, n = wl.LLAMA7B, 2, args.n
    steps = args.steps = args.steps or 50
    warmup = args.warmup = 10 if args.warmup is None else args.warmup
    t_setup = time.time()
    w = wl.layer_weights(shape, seed)
    layer = DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                        ffn=shape.ffn, kv_capacity=max(n, 64), n_max=n)
    x_host = wl.activations(shape, seed, 0, n)
    x = to_device(x_host)
    out = torch.empty_like(x)
    stream = torch.cuda.Stream()
    call = layer.prepare(x, [n], [n], out=out)
    setup_s = time.time() - t_setup
    for _ in range(warmup):
        call(stream.cuda_stream)
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        call(stream.cuda_stream)
    stream.synchronize()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps

    kernel_ms = time_steps(torch, rx, stream, lambda i: call(stream.cuda_stream), [0, 1, 2, 3, 4], min(steps, 20))
    P = sum(m * k for m, k in shape.matrices().values())
    m, k = shape.matrices()["wgu"]
    gu_flops = 2.0 * n * m * k
    ach = gu_flops / (kernel_ms["gate_up"] * 1e-3) / 1e12
    gemm_ms = kernel_ms["qkv"] + kernel_ms["o_proj"] + kernel_ms["gate_up"] + kernel_ms["down"]
    attn_flops = 4.0 * (n * (n + 1) / 2) * shape.n_heads * shape.head_dim
    kernel = ("gemm_q4_mfma_kernel<EPI_SWIGLU> (gate/up GEMM, m=22016, k=4096, n=%d)" % n if n > 64 else
              "skinny_q4_kernel + skinny_finish_kernel<EPI_SWIGLU> (gate/up, m=22016, k=4096, n=%d)" % n)
    roofline = {"bound": "mfma", "kernel": kernel, "achieved": round(ach, 1), "peak": PEAK_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(ach / PEAK_MFMA_TFLOPS, 4), "traffic": traffic_from_profile("traffic_gate_up_gemm_7b_n%d.json" % n),
                "algorithmic_flops_per_launch": gu_flops, "avg_launch_ms": round(kernel_ms["gate_up"], 5)}

    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        mats = shape.matrices()
        ow = oracle.LayerWeights(*(oracle.QMat(w[nm + ".q"], w[nm + ".s"], *mats[nm]) for nm in ("wqkv", "wo", "wgu", "wdown")),
                                 w["norm_attn"], w["norm_ffn"])
        rows = min(n, 48)                            # causal: the first rows of the call equal a shorter prefill of the same input
        od = oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.rms_eps, shape.rope_base, rows)
        cshape = (1, rows, shape.n_kv_heads, shape.head_dim)
        t1 = time.perf_counter()
        ref = oracle.decoder_layer(od, ow, x_host[:rows], np.zeros(cshape, np.float32), np.zeros(cshape, np.float32), oracle.Seqs([rows], [rows]))
        t_cpu = time.perf_counter() - t1
        got = f16_bits(out).view(np.float16).astype(np.float32)[:rows]
        err = np.abs(got - ref)
        assert np.all(err <= 1e-2 + 2e-2 * np.abs(ref)), "bench: GPU prefill rows are outside tolerance"
        cpu = {"value": round(rows / t_cpu, 3), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "prefill of the first %d rows of the same input (causal: they equal rows 0..%d of the timed call), %.1f s of "
                         "oracle time; GPU rows checked against it, max abs err %.2e" % (rows, rows - 1, t_cpu, float(err.max()))}

    emit(args, "prefill tokens/s (7B-shaped int4 layer) + MFMA utilisation", "tokens/s", n * steps / elapsed, ms_per_step,
         "f16 MFMA (int4 weights, f32 accumulate)",
         {"workload": "configs[2]: one Llama-2-7B-shaped int4-g32 decoder layer, prefill of n=%d rows, L=n, empty cache; 1 step = 1 call "
                      "(the same binary serves every n)" % n,
          "n": n, "build_id": rx.relax_build_id(), "setup_s": round(setup_s, 1)},
         roofline, cpu,
         {"kernel_ms": {k_: round(v, 5) for k_, v in kernel_ms.items()},
          "gemm_steps": {"flops": 2.0 * n * P, "ms": round(gemm_ms, 5), "TFLOPs": round(2.0 * n * P / gemm_ms / 1e9, 1),
                         "frac_of_mfma_peak": round(2.0 * n * P / gemm_ms / 1e9 / PEAK_MFMA_TFLOPS, 4),
                         "note": "qkv step includes RMSNorm and rotary/append kernels"},
          "attention": {"flops": attn_flops, "ms": round(kernel_ms["attention"], 5),
                        "TFLOPs": round(attn_flops / kernel_ms["attention"] / 1e9, 1)}})


# ------------------------------------------------------------------------------------------------ configs[3], configs[4]
def bench_model(args, np, torch, wl, rx, big):
    from paper_2311_02103_amd.runtime import DeviceModel
    V = 32000
    args.mode = args.mode or "eager"
    if big:
        shape, nl, distinct, B, cap, seed = wl.LLAMA70B, 80, min(args.sets, 4), 16, 8192, 4
        steps = args.steps = args.steps or 8
        warmup = args.warmup = 2 if args.warmup is None else args.warmup
    else:
        shape, nl, distinct, B, cap, seed = wl.LLAMA7B, 32, args.sets, 1, 512, 3
        steps = args.steps = args.steps or 256
        warmup = args.warmup = 8 if args.warmup is None else args.warmup
    if args.layers:
        nl = args.layers
    t_setup = time.time()
    print("bench: generating %d weight sets of the %s layer shape on the host" % (distinct, shape.name), file=sys.stderr, flush=True)
    host = [wl.layer_weights(shape, seed, layer=l) for l in range(distinct)]
    mt = wl.model_tensors(shape, seed, V)
    print("bench: host tensors ready after %.0f s, building the device model (%d layers)" % (time.time() - t_setup, nl), file=sys.stderr, flush=True)
    n_max = B if big else 128
    dev = DeviceModel([host[l % distinct] for l in range(nl)], mt["embedding"], mt["norm_final"], mt["lm_head"], hidden=shape.hidden,
                      n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap,
                      kv_slots=B, n_max=n_max, B_max=B)
    P = sum(m * k for m, k in shape.matrices().values())
    logits = torch.empty((B, V), dtype=torch.float16, device="cuda")
    nxt = torch.empty((B,), dtype=torch.int32, device="cuda")
    weight_bytes = nl * P * 0.5625 + V * shape.hidden * 2
    if big:
        kv = [int(v) for v in wl.uniform_lengths(seed, B, 100, 8000)]
        for l in range(nl):                         # cache contents: N(0,1) drawn on the device (parity of this shape is a test's job)
            dev.k[l].normal_()
            dev.v[l].normal_()
        ids = torch.from_numpy(wl.token_ids(seed, B, V)).cuda()
        setup_s = time.time() - t_setup
        print("bench: device model and KV caches ready after %.0f s" % setup_s, file=sys.stderr, flush=True)
        step = lambda s: dev.step(ids if s == 0 else nxt, [1] * B, [k + s for k in kv], logits=logits, next_ids=nxt)
        for s in range(warmup):
            step(s)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(warmup, warmup + steps):
            step(s)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        kv_bytes = shape.kv_bytes_per_token() * float(sum(kv) + B * (warmup + steps / 2.0)) * nl
        tokens = B * steps
        desc = ("configs[4]: Llama-2-70B-shaped GQA model (hidden 8192, 64/8 heads x 128, FFN 28672), %d layers (%d distinct int4-g32 "
                "weight sets cycled, 1.9 GB: more than the last-level cache), vocab 32000, batched decode of 16 sequences, "
                "L_b~U{100..8000} (sum %d), kv_capacity 8192; 1 step = 1 relax_model_step = 16 tokens" % (nl, distinct, sum(kv)))
        metric = "decode tokens/s (70B-shaped int4 GQA model, batch 16)"
    else:
        prompt = torch.from_numpy(wl.token_ids(seed, 128, V)).cuda()
        setup_s = time.time() - t_setup
        dev.step(prompt, [128], [128], logits=logits, next_ids=nxt)
        if args.mode == "graph":
            # Graph offloading (Sec. 4.5) over a device-resident descriptor (the shape heap of Sec. 4.7): a decode step -- a
            # one-element add that advances kv_len in the table, then relax_model_step, which reads the token from the buffer
            # it writes the next one to -- is captured, args.graph_steps times in a row, and replayed; the host passes only
            # the bound.  Nothing in the graph depends on the position, so the same graph serves every token.
            table = torch.tensor([[0], [1], [128], [0]], dtype=torch.int32, device="cuda")
            one = torch.ones((), dtype=torch.int32, device="cuda")
            gstream = torch.cuda.Stream()

            def graph_body():
                table[2].add_(one)
                dev.step(nxt, [1], [cap], logits=logits, next_ids=nxt, stream=gstream, device_table=table)

            gs = max(1, args.graph_steps)
            if steps % gs != 0:
                raise SystemExit("bench: --steps must be a multiple of --graph-steps")
            with torch.cuda.stream(gstream):
                graph_body()                              # everything touched once before capture (this is decode step 0)
            gstream.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=gstream):
                for _ in range(gs):
                    graph_body()
            wrep = (max(warmup, 1) - 1 + gs - 1) // gs
            with torch.cuda.stream(gstream):
                for s in range(wrep):
                    graph.replay()
            gstream.synchronize()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            with torch.cuda.stream(gstream):
                for s in range(steps // gs):
                    graph.replay()
            gstream.synchronize()
            elapsed = time.perf_counter() - t0
            assert int(table[2].item()) == 128 + 1 + wrep * gs + steps
        else:
            for s in range(warmup):
                dev.step(nxt, [1], [129 + s], logits=logits, next_ids=nxt)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for s in range(warmup, warmup + steps):
                dev.step(nxt, [1], [129 + s], logits=logits, next_ids=nxt)
            torch.cuda.synchronize()
            elapsed = time.perf_counter() - t0
        kv_bytes = shape.kv_bytes_per_token() * (129 + warmup + steps / 2.0) * nl
        tokens = steps
        desc = ("configs[3]: %d-layer Llama-2-7B-shaped model (%d distinct int4-g32 weight sets cycled), fp16 embedding and LM head, "
                "vocab 32000, 128-token random-id prompt, then greedy decode at batch 1 (next id fed back on the device); "
                "1 step = 1 relax_model_step = 1 token" % (nl, distinct))
        metric = "decode tokens/s (7B-shaped int4 model, batch 1)"
    ms_per_step = elapsed * 1e3 / steps
    step_bytes = weight_bytes + kv_bytes
    model_gbs = step_bytes / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: the gate/up matmul of a layer, bracketed by the ABI's hook inside the model step
    stream = torch.cuda.current_stream()
    if big:
        tcall = lambda i: dev.step(ids, [1] * B, kv, logits=logits, next_ids=nxt)
    else:
        tcall = lambda i: dev.step(nxt, [1], [129 + warmup + steps], logits=logits, next_ids=nxt)
    kernel_ms = time_steps(torch, rx, stream, tcall, [3], 10)
    m, k = shape.matrices()["wgu"]
    gu_bytes = m * (k // 2) + m * (k // 32) * 2
    ach = gu_bytes / (kernel_ms["gate_up"] * 1e-3) / 1e9
    kernel = ("skinny_q4_kernel<1,16> + skinny_finish_kernel<EPI_SWIGLU> (gate/up, m=57344, k=8192, n=16)" if big else
              "gemv_q4_reg_kernel<X_F32_NORM, EPI_SWIGLU, 2> (gate/up matvec, m=22016, k=4096)")
    roofline = {"bound": "hbm", "kernel": kernel, "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": round(ach / PEAK_HBM_GBS, 4),
                "traffic": traffic_from_profile("traffic_gate_up_skinny_70b.json" if big else "traffic_gate_up_matvec_7b.json"),
                "algorithmic_bytes_per_launch": gu_bytes, "avg_launch_ms": round(kernel_ms["gate_up"], 5)}

    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        mats = shape.matrices()
        ow = oracle.LayerWeights(*(oracle.QMat(host[0][nm + ".q"], host[0][nm + ".s"], *mats[nm]) for nm in ("wqkv", "wo", "wgu", "wdown")),
                                 host[0]["norm_attn"], host[0]["norm_ffn"])
        ocap = 16
        od = oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.rms_eps, shape.rope_base, ocap)
        cshape = (B, ocap, shape.n_kv_heads, shape.head_dim)
        Ko, Vo = np.zeros(cshape, np.float32), np.zeros(cshape, np.float32)
        xs = wl.activations(shape, seed, 7, B)
        t_cpu, done = 0.0, 0
        while t_cpu < args.cpu_seconds and done < ocap:
            t1 = time.perf_counter()
            oracle.decoder_layer(od, ow, xs, Ko, Vo, oracle.Seqs([1] * B, [done + 1] * B))
            t_cpu += time.perf_counter() - t1
            done += 1
        t1 = time.perf_counter()
        y = oracle.rmsnorm(wl.f16_bits_to_f32(xs), mt["norm_final"], shape.rms_eps)
        oracle.argmax(oracle.half_matmul(y, mt["lm_head"]))
        t_head = time.perf_counter() - t1
        per_step = nl * t_cpu / done + t_head
        cpu = {"value": round(B / per_step, 4), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "EXTRAPOLATED: %d calls of one layer of this shape on %d decode rows (short KV lengths) took %.1f s, the LM head "
                         "+ final norm + argmax %.2f s; a model step is taken as %d x the layer time + the head (parity of this "
                         "workload is covered by the teacher-forced tests, not here)" % (done, B, t_cpu, t_head, nl)}

    emit(args, metric, "tokens/s", tokens / elapsed, ms_per_step, "f16 (int4 weights, f32 accumulate)",
         {"workload": desc, "build_id": rx.relax_build_id(), "setup_s": round(setup_s, 1), "launch": ("hipGraph of %d decode steps (descriptor on the device), captured once and replayed" % max(1, args.graph_steps) if (not big and args.mode == "graph")
                                                                                     else "eager (one C call per step)")},
         roofline, cpu,
         {"model_hbm": {"algorithmic_bytes_per_step": int(step_bytes), "weights_and_head_bytes": int(weight_bytes), "kv_bytes": int(kv_bytes),
                        "achieved_GBps": round(model_gbs, 1), "frac_of_peak": round(model_gbs / PEAK_HBM_GBS, 4)},
          "us_per_layer": round(ms_per_step * 1e3 / nl, 2), "kernel_ms": {k_: round(v, 5) for k_, v in kernel_ms.items()}})


# ------------------------------------------------------------------------------------------------ batch sweep
def bench_batch_sweep(args, np, torch, wl, rx):
    """One 7B-shaped layer call on n decode rows (n sequences, one row each, 256 cached tokens each) against n: where the
    runtime dispatch on the symbolic row count (Sec. 5.1) changes kernels -- matvec kernels for one row (and up to four rows
    of a model this small, two or four rows of x per pass over the weights), the few-row MFMA kernel up to 128 rows (64 for the
    tall gate/up matrix), the tiled GEMM above."""
    from paper_2311_02103_amd.runtime import DeviceLayer, to_device
    shape, seed, cap, L = wl.LLAMA7B, 6, 320, 256
    ns = [int(v) for v in args.sweep_rows.split(",")] if args.sweep_rows else [1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 65, 96, 128, 129, 192, 256]
    steps = args.steps = args.steps or 60
    warmup = args.warmup = 10 if args.warmup is None else args.warmup
    sets = max(1, min(args.sets, 3))                # three sets = 342 MB of weights: more than the last-level cache
    layers = []
    for s_ in range(sets):
        layers.append(DeviceLayer(wl.layer_weights(shape, seed, layer=s_), hidden=shape.hidden, n_heads=shape.n_heads,
                                  n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap,
                                  kv_slots=max(ns), n_max=max(ns), B_max=max(ns), share_from=layers[0] if layers else None))
        layers[-1].k.normal_()
        layers[-1].v.normal_()
    stream = torch.cuda.Stream()
    rows = []
    for n in ns:
        x = to_device(wl.activations(shape, seed, n, n))
        out = torch.empty_like(x)
        calls = [lay.prepare(x, [1] * n, [L] * n, out=out) for lay in layers]
        for i in range(warmup):
            calls[i % sets](stream.cuda_stream)
        stream.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            calls[i % sets](stream.cuda_stream)
        stream.synchronize()
        us = (time.perf_counter() - t0) * 1e6 / steps
        matmuls = ("matvec" if n == 1 else "matvec, 2 or 4 rows per pass" if n <= 4 else "few-row MFMA" if n <= 64 else
                   "few-row MFMA, tiled GEMM for gate/up" if n <= 128 else "tiled GEMM")
        rows.append({"n": n, "us_per_call": round(us, 1), "layer_tokens_per_s": round(n / us * 1e6, 0), "matmul_kernels": matmuls})
    best = max(rows, key=lambda r: r["layer_tokens_per_s"])
    emit(args, "layer-tokens/s of one 7B-shaped int4 layer call against the number of decode rows (best point)", "tokens/s",
         best["layer_tokens_per_s"], best["us_per_call"] / 1e3, "f16 (int4 weights, f32 accumulate)",
         {"workload": "batch sweep on the int4 path (the paper sweeps batch sizes in Sec. 5.1): n decode rows, one per sequence, L = 256, %d rotating weight sets" % sets,
          "build_id": rx.relax_build_id()}, None, None, {"batch_sweep": rows})


# ------------------------------------------------------------------------------------------------ one decode row at three model shapes
def bench_decode_shapes(args, np, torch, wl, rx):
    """One decode row (n = 1, 2231 cached tokens) through one int4 layer of the 7B, 13B and 70B shapes of the paper's LLM
    evaluation (Sec. 5.1): the same binary, the dispatch on k picks the chunk count of the matvec, the long-row kernel for
    the down projections of 13B / 70B, the grouped-query attention kernel for 70B.  Weight codes and scales are random
    bits made on the device (the time does not depend on them); graph replays over rotating weight sets."""
    from paper_2311_02103_amd.runtime import DeviceLayer
    L = 2231
    steps = args.steps = args.steps or 10
    args.warmup = 1 if args.warmup is None else args.warmup
    shapes = [(wl.LLAMA7B, 8), (wl.LayerShape("llama2-13b", hidden=5120, n_heads=40, n_kv_heads=40, head_dim=128, ffn=13824), 6), (wl.LLAMA70B, 3)]
    rs = np.random.RandomState(12)
    rows = []
    for shape, sets in shapes:
        layers = []
        for _ in range(sets):
            w = {}
            for name, (m, k) in shape.matrices().items():
                w[name + ".q"] = rs.randint(0, 2 ** 31 - 1, size=(m, k // 8)).astype(np.int32)
                w[name + ".s"] = (rs.rand(m, k // 32) * 0.004 + 0.002).astype(np.float16).view(np.uint16)
            w["norm_attn"] = np.ones(shape.hidden, np.float16).view(np.uint16)
            w["norm_ffn"] = np.ones(shape.hidden, np.float16).view(np.uint16)
            lay = DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim,
                              ffn=shape.ffn, kv_capacity=L, kv_slots=1, n_max=1, B_max=1)
            lay.k.normal_()
            lay.v.normal_()
            layers.append(lay)
        x = (torch.randn(1, shape.hidden, device="cuda") * 0.5).half()
        calls = [lay.prepare(x, [1], [L]) for lay in layers]
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            for c in calls:
                c(st.cuda_stream)
            st.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=st):
                for _ in range(4):
                    for c in calls:
                        c(st.cuda_stream)
            for _ in range(args.warmup):
                g.replay()
            st.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(st)
            for _ in range(steps):
                g.replay()
            e1.record(st)
            st.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / (steps * 4 * sets)
        nbytes = sum(m * k * (0.5 + 2 / 32) for m, k in shape.matrices().values()) + 2 * L * shape.n_kv_heads * shape.head_dim * 2
        rows.append({"shape": shape.name, "us_per_call": round(us, 2), "algorithmic_MB": round(nbytes / 1e6, 1),
                     "GBps": round(nbytes / us / 1e3, 1), "frac_of_hbm_peak": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4)})
        del layers, calls, g
        torch.cuda.empty_cache()
    head = rows[0]
    emit(args, "decode layer calls/s at one row (7B shape; 13B and 70B shapes in decode_shapes)", "calls/s", 1e6 / head["us_per_call"],
         head["us_per_call"] / 1e3, "f16 (int4 weights, f32 accumulate)",
         {"workload": "one decode row, L = %d, one int4-g32 layer of the 7B / 13B / 70B shapes, graph replays over rotating weight sets" % L,
          "build_id": rx.relax_build_id()},
         {"bound": "hbm", "kernel": "the five (13B) or six (70B: grouped-query attention + merge) launches of the one-row layer",
          "achieved": head["GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": head["frac_of_hbm_peak"], "traffic": None}, None, {"decode_shapes": rows})


# ------------------------------------------------------------------------------------------------ fp16-weight sweep
def bench_half_sweep(args, np, torch, wl, rx):
    """relax_half_matmul (plain fp16 weights) against the row count n on two 7B-shaped matrices, with the matvec passes and the
    tiled GEMM forced in turn: where the matrix-vector form stops paying (Sec. 5.1 of the paper: its LLM charts sweep the batch
    size on fp16 weights).  Weight copies are rotated so that each launch streams its matrix from HBM."""
    steps = args.steps = args.steps or 30
    warmup = args.warmup = 5 if args.warmup is None else args.warmup
    ns = [1, 2, 4, 8, 9, 10, 12, 16, 24, 32, 64, 128, 256, 512, 1024, 2048]
    stream = torch.cuda.Stream()
    table = {}
    try:
        for name, (m, k) in (("o_proj 4096x4096", (4096, 4096)), ("gate_up 22016x4096", (22016, 4096))):
            copies = max(3, int(600e6 // (m * k * 2)))
            ws_ = [(torch.randn((m, k), device="cuda", dtype=torch.float32) * 0.02).to(torch.float16) for _ in range(copies)]
            rows = []
            x = torch.randn((8, k), device="cuda", dtype=torch.float16)
            out = torch.empty((8, m), dtype=torch.float16, device="cuda")
            for i in range(4 * copies):                   # first touches of the fresh copies (address translation) stay out of the sweep
                rx.check(rx.relax_half_matmul(x, ws_[i % copies], out, 8, m, k, stream))
            stream.synchronize()
            for n in ns:
                x = torch.randn((n, k), device="cuda", dtype=torch.float16)
                out = torch.empty((n, m), dtype=torch.float16, device="cuda")
                res = {"n": n}
                for label, gemm_rows in (("matvec_us", 10 ** 6), ("gemm_us", 1)):
                    if label == "matvec_us" and n > 64:
                        continue                        # n / 8 passes over the matrix: far off by then
                    rx.check(rx.relax_set_option("half_matmul_gemm_rows", gemm_rows))
                    for i in range(warmup):
                        rx.check(rx.relax_half_matmul(x, ws_[i % copies], out, n, m, k, stream))
                    stream.synchronize()
                    t0 = time.perf_counter()
                    for i in range(steps):
                        rx.relax_half_matmul(x, ws_[i % copies], out, n, m, k, stream)
                    stream.synchronize()
                    res[label] = round((time.perf_counter() - t0) * 1e6 / steps, 1)
                rows.append(res)
            both = [r for r in rows if "matvec_us" in r]
            cross = next((r["n"] for r in both if r["gemm_us"] < r["matvec_us"]), None)
            table[name] = {"rows": rows, "gemm_faster_from_n": cross, "weight_MB": round(m * k * 2 / 1e6, 1)}
            del ws_
    finally:
        rx.check(rx.relax_set_option("half_matmul_gemm_rows", 0))     # back to the default: by estimate
    # the whole 7B-shaped layer on fp16 weights (relax_decoder_layer_f16: eleven launches), three rotating weight sets of 405 MB
    layer16 = {}
    shape7 = wl.LLAMA7B
    dims = rx.make_dims(shape7.hidden, shape7.n_heads, shape7.n_kv_heads, shape7.head_dim, shape7.ffn, 2304, 1, shape7.rms_eps, shape7.rope_base, 32)
    sets16 = []
    for _ in range(3):
        mats = [(torch.randn((m, k), device="cuda", dtype=torch.float32) * 0.02).to(torch.float16)
                for m, k in ((12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008))]
        nw = (torch.randn(4096, device="cuda") * 0.1 + 1.0).to(torch.float16)
        sets16.append(mats + [nw, nw])
    rope = torch.empty(rx.relax_rope_table_bytes(dims) // 4, dtype=torch.float32, device="cuda")
    rx.check(rx.relax_rope_table_init(dims, rope, stream), "relax_rope_table_init")
    kc = torch.randn((1, 2304, shape7.n_kv_heads, shape7.head_dim), device="cuda", dtype=torch.float16)
    cache = rx.KVCache(kc, kc.clone(), rope)
    wbytes = 2 * (12288 * 4096 + 4096 * 4096 + 22016 * 4096 + 4096 * 11008)
    for n, L, reps in ((1, 2231, 120), (2048, 2048, 6)):
        wsb = rx.relax_layer_f16_workspace_bytes(dims, n, 2304, 1)
        ws16 = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        x16 = torch.randn((n, 4096), device="cuda", dtype=torch.float16)
        o16 = torch.empty_like(x16)
        seqs = rx.Seqs([n], [L], None, None)
        for i in range(6):
            rx.check(rx.relax_decoder_layer_f16(dims, sets16[i % 3], x16, cache, seqs, o16, n, ws16, wsb, stream), "relax_decoder_layer_f16")
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        stream.synchronize()
        start.record(stream)
        for i in range(reps):
            rx.relax_decoder_layer_f16(dims, sets16[i % 3], x16, cache, seqs, o16, n, ws16, wsb, stream)
        stop.record(stream)
        stream.synchronize()
        us = start.elapsed_time(stop) * 1e3 / reps
        row = {"us_per_call": round(us, 1)}
        if n == 1:
            alg = wbytes + 2 * L * shape7.n_kv_heads * shape7.head_dim * 2
            row.update(algorithmic_MB=round(alg / 1e6, 1), GBps=round(alg / us / 1e3, 1), frac_of_hbm_peak=round(alg / us / 1e3 / PEAK_HBM_GBS, 4))
        layer16["n=%d L=%d" % (n, L)] = row
        del ws16, x16, o16
    del sets16, kc, cache
    big = table["gate_up 22016x4096"]["rows"][-1]
    tflops = 2.0 * 2048 * 22016 * 4096 / (big["gemm_us"] * 1e-6) / 1e12
    emit(args, "fp16-weight GEMM rate at n = 2048 on the gate/up shape (22016 x 4096)", "TFLOP/s", tflops, big["gemm_us"] / 1e3, "f16 MFMA, f32 accumulate",
         {"workload": "fp16-weight matmul against the row count, matvec passes and tiled GEMM forced in turn", "build_id": rx.relax_build_id()},
         {"bound": "mfma", "kernel": "gemm_q4_mfma_kernel<EPI_F16, 4, 4, fp16 weights>", "achieved": round(tflops, 1), "peak": PEAK_MFMA_TFLOPS,
          "unit": "TFLOP/s", "frac": round(tflops / PEAK_MFMA_TFLOPS, 4), "traffic": None}, None, {"half_sweep": table, "f16_layer_7b": layer16})


# ------------------------------------------------------------------------------------------------ 3-bit matvec
def bench_q3_matvec(args, np, torch, wl, rx):
    """relax_dequant_matmul_q3_native (and, beside it, relax_dequant_matmul_q3 on the canonical stream) at n = 1 on the four matrix shapes of the 7B layer (Sec. 5.3 of the paper deploys 3-bit models):
    HIP-event time per launch on the launch stream over rotating weight copies (each launch streams its matrix from HBM),
    algorithmic bytes = 3-bit codes + fp16 scales + x + out.  The CPU leg times the numpy reference on a row sample of the
    gate/up matrix and checks the GPU's outputs for those rows against it."""
    steps = args.steps = args.steps or 400
    warmup = args.warmup = 40 if args.warmup is None else args.warmup
    stream = torch.cuda.Stream()
    table, keep = {}, None
    for name, (m, k) in (("gate_up 22016x4096", (22016, 4096)), ("qkv 12288x4096", (12288, 4096)), ("down 4096x11008", (4096, 11008)),
                         ("o_proj 4096x4096", (4096, 4096))):
        wbytes = m * k * 3 // 8 + m * (k // 32) * 2
        copies = max(3, int(600e6 // wbytes))
        qs = [torch.randint(-2 ** 31, 2 ** 31 - 1, (m, 3 * k // 32), dtype=torch.int32, device="cuda") for _ in range(copies)]
        ss = [(torch.rand((m, k // 32), device="cuda") * 0.01 + 0.002).to(torch.float16) for _ in range(copies)]
        mats = [rx.QMat(q, s, m, k) for q, s in zip(qs, ss)]
        nqs = [torch.empty_like(q) for q in qs]
        for mat, nq in zip(mats, nqs):
            rx.check(rx.relax_repack_q3(mat, nq, stream), "relax_repack_q3")
        nmats = [rx.QMat(nq, s, m, k) for nq, s in zip(nqs, ss)]
        x = torch.randn((1, k), device="cuda", dtype=torch.float16)
        out = torch.empty((1, m), dtype=torch.float16, device="cuda")
        alg = wbytes + k * 2 + m * 2
        row = {"algorithmic_MB": round(alg / 1e6, 2), "weight_copies": copies}
        for layout, fn, ms_ in (("native", rx.relax_dequant_matmul_q3_native, nmats), ("canonical", rx.relax_dequant_matmul_q3, mats)):
            for i in range(warmup + 2 * copies):
                rx.check(fn(x, ms_[i % copies], out, 1, stream))
            start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            stream.synchronize()
            start.record(stream)
            for i in range(steps):
                fn(x, ms_[i % copies], out, 1, stream)
            stop.record(stream)
            stream.synchronize()
            us = start.elapsed_time(stop) * 1e3 / steps
            row[layout] = {"us_per_launch": round(us, 2), "GBps": round(alg / us / 1e3, 1), "frac_of_peak": round(alg / us / 1e3 / PEAK_HBM_GBS, 4)}
        table[name] = row
        if keep is None:
            outs = []
            for fn, mat in ((rx.relax_dequant_matmul_q3_native, nmats[0]), (rx.relax_dequant_matmul_q3, mats[0])):
                rx.check(fn(x, mat, out, 1, stream))
                stream.synchronize()
                outs.append(out[0, :2048].float().cpu().numpy())
            keep = (m, k, qs[0][:2048].cpu().numpy().view(np.uint32), ss[0][:2048].cpu().numpy().view(np.uint16),
                    x.cpu().numpy().astype(np.float32), outs)
        del qs, ss, mats, nqs, nmats
    # the same format at n = 2048: from 16 rows on the native-layout call goes through the tiled MFMA GEMM
    gemm = {}
    for name, (m, k) in (("gate_up 22016x4096", (22016, 4096)), ("qkv 12288x4096", (12288, 4096)), ("down 4096x11008", (4096, 11008)),
                         ("o_proj 4096x4096", (4096, 4096))):
        n = 2048
        nq = torch.randint(-2 ** 31, 2 ** 31 - 1, (m, 3 * k // 32), dtype=torch.int32, device="cuda")
        sc = (torch.rand((m, k // 32), device="cuda") * 0.01 + 0.002).to(torch.float16)
        xb = torch.randn((n, k), device="cuda", dtype=torch.float16)
        ob = torch.empty((n, m), dtype=torch.float16, device="cuda")
        mat = rx.QMat(nq, sc, m, k)
        for _ in range(3):
            rx.check(rx.relax_dequant_matmul_q3_native(xb, mat, ob, n, stream))
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        stream.synchronize()
        start.record(stream)
        for _ in range(20):
            rx.relax_dequant_matmul_q3_native(xb, mat, ob, n, stream)
        stop.record(stream)
        stream.synchronize()
        us = start.elapsed_time(stop) * 1e3 / 20
        gemm[name] = {"us_per_launch": round(us, 1), "TFLOPs": round(2.0 * n * m * k / us / 1e6, 1), "frac_of_mfma_peak": round(2.0 * n * m * k / us / 1e6 / PEAK_MFMA_TFLOPS, 4)}
        del nq, sc, xb, ob, mat
    # the whole 7B-shaped layer on 3-bit weights (relax_decoder_layer_q3: eleven launches, nothing fused), three rotating weight sets
    layer3 = {}
    shape7 = wl.LLAMA7B
    dims = rx.make_dims(shape7.hidden, shape7.n_heads, shape7.n_kv_heads, shape7.head_dim, shape7.ffn, 2304, 1, shape7.rms_eps, shape7.rope_base, 32)
    sets3 = []
    for _ in range(3):
        qm = []
        for m, k in ((12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008)):
            nq = torch.randint(-2 ** 31, 2 ** 31 - 1, (m, 3 * k // 32), dtype=torch.int32, device="cuda")
            sc = (torch.rand((m, k // 32), device="cuda") * 0.01 + 0.002).to(torch.float16)
            qm.append(rx.QMat(nq, sc, m, k, 32))
        nw = (torch.randn(4096, device="cuda") * 0.1 + 1.0).to(torch.float16)
        sets3.append(rx.LayerWeights(*qm, nw, nw))
    rope = torch.empty(rx.relax_rope_table_bytes(dims) // 4, dtype=torch.float32, device="cuda")
    rx.check(rx.relax_rope_table_init(dims, rope, stream), "relax_rope_table_init")
    kc = torch.randn((1, 2304, shape7.n_kv_heads, shape7.head_dim), device="cuda", dtype=torch.float16)
    cache = rx.KVCache(kc, kc.clone(), rope)
    for n, L, reps in ((1, 2231, 120), (2048, 2048, 6)):
        wsb = rx.relax_layer_q3_workspace_bytes(dims, n, 2304, 1)
        ws3 = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        x3 = torch.randn((n, 4096), device="cuda", dtype=torch.float16)
        o3 = torch.empty_like(x3)
        seqs = rx.Seqs([n], [L], None, None)
        for i in range(6):
            rx.check(rx.relax_decoder_layer_q3(dims, sets3[i % 3], x3, cache, seqs, o3, n, ws3, wsb, stream), "relax_decoder_layer_q3")
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        stream.synchronize()
        start.record(stream)
        for i in range(reps):
            rx.relax_decoder_layer_q3(dims, sets3[i % 3], x3, cache, seqs, o3, n, ws3, wsb, stream)
        stop.record(stream)
        stream.synchronize()
        layer3["n=%d L=%d" % (n, L)] = {"us_per_call": round(start.elapsed_time(stop) * 1e3 / reps, 1)}
        del ws3, x3, o3
    del sets3, kc, cache
    cpu = None
    if args.cpu_seconds > 0:
        from oracle import q3                               # the CPU reference: baseline and check only
        m, k, qh, sh, xh, got = keep
        reps, t0 = 0, time.perf_counter()
        while reps < 1 or time.perf_counter() - t0 < min(args.cpu_seconds, 10.0):
            ref = q3.dequant_matmul_q3(xh, qh, sh, 2048, k)[0]
            reps += 1
        sec = (time.perf_counter() - t0) / reps
        for one in got:                                     # native layout (repacked from the same codes), then canonical
            err = np.abs(one - ref)
            assert np.all(err <= 1e-2 + 2e-2 * np.abs(ref)), "3-bit matvec differs from the reference: max err %g" % err.max()
        sample_bytes = 2048 * (k * 3 // 8 + (k // 32) * 2)
        cpu = {"value": round(sample_bytes / sec / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": "rows 0..2047 of the gate/up matrix, %d repetitions of the numpy reference (%.2f s each); the GPU's outputs for those rows checked against it" % (reps, sec)}
    g = dict(table["gate_up 22016x4096"]["native"], algorithmic_MB=table["gate_up 22016x4096"]["algorithmic_MB"])
    emit(args, "3-bit matvec, algorithmic GB/s on the 7B gate/up shape (22016 x 4096, n = 1)", "GB/s", g["GBps"], g["us_per_launch"] / 1e3,
         "f16 (3-bit weights, f32 accumulate)",
         {"workload": "3-bit group-32 weights in the native word layout (repacked once from the canonical stream), n = 1, the four matrix shapes of the 7B layer, rotating weight copies; the canonical-layout kernel timed beside it", "build_id": rx.relax_build_id()},
         {"bound": "hbm", "kernel": "gemv_q3n_kernel (22016 x 4096)", "achieved": g["GBps"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
          "frac": g["frac_of_peak"], "traffic": None, "algorithmic_bytes_per_launch": int(g["algorithmic_MB"] * 1e6), "avg_launch_ms": g["us_per_launch"] / 1e3},
         cpu, {"q3_matvec": table, "q3_gemm_n2048": gemm, "q3_layer_7b": layer3})


# ------------------------------------------------------------------------------------------------ memory plan
def bench_memory_plan(args, wl, rx):
    """The shape of the paper's activation-memory experiment (Sec. 5: prefill of 128..1024 tokens, decode at batch 1..64,
    with and without static planning), on the layer workspace of this library: bytes of the intermediates when every
    tensor and every kernel workspace has its own allocation, against the plan of Alg. 3 (relax_workspace_plan)."""
    args.steps, args.warmup = args.steps or 1, args.warmup or 0
    table = {}
    for shape in (wl.LLAMA7B, wl.LLAMA70B):
        cap = 8192
        dims = rx.make_dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, cap, 64)
        rows = []
        for kind, cases in (("prefill", [(n, n, 1) for n in (128, 256, 512, 1024)]), ("decode", [(b, 4096, b) for b in (1, 16, 32, 64)])):
            for n, L, B in cases:
                rc, entries, planned, unplanned = rx.relax_workspace_plan(dims, n, L, B)
                rx.check(rc, "relax_workspace_plan")
                rc, entries_eq, planned_eq, _ = rx.relax_workspace_plan(dims, n, L, B, rule=1)
                rx.check(rc, "relax_workspace_plan_rule")
                rows.append({"case": "%s n=%d L=%d B=%d" % (kind, n, L, B), "unplanned_bytes": unplanned,
                             "planned_bytes_equal_rule": planned_eq, "ratio_equal_rule": round(planned_eq / unplanned, 4),
                             "storages_equal_rule": len({e["storage"] for e in entries_eq}),
                             "planned_bytes": planned, "ratio": round(planned / unplanned, 4),
                             "storages": len({e["storage"] for e in entries}), "tensors": len(entries)})
        table[shape.name] = rows
    head = table[wl.LLAMA7B.name][3]
    emit(args, "planned / unplanned activation bytes of one layer call (7B shape, prefill of 1024 tokens)", "ratio", head["ratio"], 0.0,
         "bytes", {"workload": "dynamic shape-aware memory planning (Sec. 4.3, Alg. 3) of the layer workspace, in the shape of the paper's activation-memory experiment "
                               "(Sec. 5.2: prefill 128..1024, decode batch 1..64); *_equal_rule = the paper's rule (reuse on proven-equal symbolic sizes), "
                               "the unsuffixed columns = the library's layout rule (reuse when the request provably fits); host-only, nothing is timed",
                   "build_id": rx.relax_build_id()}, None, None, {"higher_is_better": False, "memory_plan": table})


# ------------------------------------------------------------------------------------------------ device ceilings
def bench_ceilings(args, np, torch, wl, rx):
    """What the device at hand reaches on a plain streaming read (1 GiB, two buffers alternated: more than the
    last-level cache) and on a bare MFMA loop: the measured-achievable counterparts of the two published peaks."""
    steps = args.steps = args.steps or 20
    args.warmup = 2 if args.warmup is None else args.warmup
    sink = torch.zeros(256 * 1024, dtype=torch.float32, device="cuda")
    bufs = [torch.full((256 * 1024 * 1024,), 1.0, dtype=torch.float32, device="cuda") for _ in range(2)]
    nbytes = bufs[0].numel() * 4

    def timed(fn, reps):
        for i in range(args.warmup):
            fn(i)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(reps):
            fn(i)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    ms_read = timed(lambda i: rx.check(rx.relax_probe_stream_read(bufs[i % 2], nbytes, sink)), steps)
    out = {}
    for name, rnd in (("near_constant_operands", False), ("random_operands", True)):
        flops = [0]

        def call(i):
            rc, flops[0] = rx.relax_probe_mfma(sink, 4000, rnd)
            rx.check(rc)
        ms = timed(call, 5)
        out[name] = round(flops[0] / ms / 1e9, 1)
    ach = nbytes / ms_read / 1e6
    # Chain of dependent launches that only stream (one stream, captured in a graph, every launch on memory that has
    # not been touched for 2 GiB): what a launch of the decode layer costs before any arithmetic, as a fixed part per
    # launch plus bytes over a streaming rate.
    stream = torch.cuda.Stream()
    chain = {}
    for mb in (0, 12, 48, 96):
        nb, nl = max(mb << 20, 4096), 48
        ptrs = [bufs[j % 2].data_ptr() + ((j // 2) * (96 << 20)) % (nbytes - (96 << 20)) for j in range(nl)]
        with torch.cuda.stream(stream):
            rx.check(rx.relax_probe_stream_read(ptrs[0], nb, sink, stream=stream))
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for j in range(nl):
                rx.check(rx.relax_probe_stream_read(ptrs[j], nb, sink, stream=stream))
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(stream):
            g.replay()
            a.record(stream)
            for _ in range(10):
                g.replay()
            b.record(stream)
        stream.synchronize()
        chain["%d MB" % mb] = round(a.elapsed_time(b) * 1e3 / (10 * nl), 2)
    slope = (96 - 48) * (1 << 20) / ((chain["96 MB"] - chain["48 MB"]) * 1e-6) / 1e9
    chain_out = {"us_per_dependent_launch": chain, "fixed_us": chain["0 MB"], "slope_GBps": round(slope, 1)}
    # The vendor's fp16 GEMM (torch.matmul, i.e. hipBLASLt / rocBLAS: fp16 weights, no decode) on the four matrix shapes of the
    # 7B layer at n = 2048 and on 8192^3, with normally distributed and with all-zero operands: the matrix pipes of this
    # chip clock down with the bit activity of their operands, so the second figure is not reachable on real data.  Context
    # for the tiled int4 GEMM only; nothing of the product calls it.
    del bufs
    torch.manual_seed(0)
    vendor = {}
    for name, (n, m, k) in (("gate_up 22016x4096", (2048, 22016, 4096)), ("qkv 12288x4096", (2048, 12288, 4096)), ("down 4096x11008", (2048, 4096, 11008)),
                            ("o_proj 4096x4096", (2048, 4096, 4096)), ("square 8192", (8192, 8192, 8192))):
        row = {}
        for kind in ("normal", "zeros"):
            if kind == "normal":
                xa = torch.randn(n, k, device="cuda", dtype=torch.float16)
                wa = (torch.randn(m, k, device="cuda") * 0.02).to(torch.float16)
            else:
                xa, wa = torch.zeros(n, k, device="cuda", dtype=torch.float16), torch.zeros(m, k, device="cuda", dtype=torch.float16)
            ms = timed(lambda i: torch.matmul(xa, wa.t()), 20)
            row[kind] = {"us": round(ms * 1e3, 1), "TFLOPs": round(2.0 * n * m * k / ms / 1e9, 1)}
        vendor[name] = row
    emit(args, "device ceilings: streaming read GB/s, MFMA loop TFLOP/s", "GB/s", ach, ms_read, "u32x4 loads / f16 MFMA",
         {"workload": "ceilings: relax_probe_stream_read over 1 GiB (two buffers alternated) and relax_probe_mfma (16 independent "
                      "32x32x16 f16 MFMAs per wavefront and iteration, 4 wavefronts per CU, 4000 iterations)", "build_id": rx.relax_build_id()},
         {"bound": "hbm", "kernel": "stream_read_kernel", "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
          "frac": round(ach / PEAK_HBM_GBS, 4), "traffic": None},
         None, {"mfma_loop_TFLOPs": out, "mfma_published_peak_TFLOPs": PEAK_MFMA_TFLOPS, "stream_chain": chain_out,
                "vendor_fp16_gemm_n2048": vendor})


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default: 1280 decode_layer, 50 prefill_layer, 256 model_7b, 8 batched_70b)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", choices=["decode_layer", "prefill_layer", "model_7b", "batched_70b", "ceilings", "memory_plan", "batch_sweep", "half_sweep", "q3_matvec", "decode_shapes"],
                    default="decode_layer")
    ap.add_argument("--n", type=int, default=2048, help="rows of the prefill_layer workload")
    ap.add_argument("--sweep-rows", default="", help="batch_sweep: comma-separated row counts instead of the default list (short profiling runs)")
    ap.add_argument("--layers", type=int, default=0, help="model workloads: override the layer count (short profiling runs)")
    ap.add_argument("--sets", type=int, default=8, help="distinct weight sets rotated through")
    ap.add_argument("--mode", choices=["graph", "eager"], default=None,
                    help="decode_layer (default graph): the 64-call schedule is captured once in a HIP graph and replayed (Sec. 4.5 of "
                         "the paper); model_7b (default eager, the faster of the two there): graph = --graph-steps decode steps captured "
                         "once over a device-resident descriptor and replayed")
    ap.add_argument("--graph-steps", type=int, default=8, help="model_7b, graph mode: decode steps captured in the one graph that is replayed")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the CPU-oracle baseline leg (0 = skip)")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="decode_layer: skip the short prefill (n = 2048) and 32-layer model runs behind the "
                                                             "`prefill` and `model_7b` keys of the line")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="before the workload, copy a 512 MiB buffer four times with a plain device copy kernel: a dispatch of known "
                         "traffic (512 MiB read, 512 MiB written) that scales rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as wl
    from paper_2311_02103_amd import binding as rx

    rx.lib()                                        # raises when the HIP library is not built: there is no fallback
    if args.workload == "memory_plan":              # host-only: the plan is a pure function of the shapes
        bench_memory_plan(args, wl, rx)
        return
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.pmc_calibration:
        src = torch.full((128 * 1024 * 1024,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.workload == "decode_layer":
        bench_decode_layer(args, np, torch, wl, rx)
    elif args.workload == "prefill_layer":
        bench_prefill_layer(args, np, torch, wl, rx)
    elif args.workload == "ceilings":
        bench_ceilings(args, np, torch, wl, rx)
    elif args.workload == "batch_sweep":
        bench_batch_sweep(args, np, torch, wl, rx)
    elif args.workload == "half_sweep":
        bench_half_sweep(args, np, torch, wl, rx)
    elif args.workload == "q3_matvec":
        bench_q3_matvec(args, np, torch, wl, rx)
    elif args.workload == "decode_shapes":
        bench_decode_shapes(args, np, torch, wl, rx)
    else:
        bench_model(args, np, torch, wl, rx, big=args.workload == "batched_70b")


if __name__ == "__main__":
    main()
