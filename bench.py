#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

Workload (configs[1] of the benchmark spec): one Llama-2-7B-shaped int4 (group 32) decoder layer,
batch 1, n = 1, KV length L drawn uniformly from 1..4096 for each of 64 calls (seeded), fp16 KV
cache pre-filled with N(0,1).  A step is one call of relax_decoder_layer = one token through one
layer.  Consecutive steps use different weight sets (8 sets, 911 MB in total) so the 256 MB
last-level cache cannot hold the weights and the packed int4 stream really comes from HBM.

Prints ONE JSON line (see README for the field meanings).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
STEP_NAMES = ["qkv_matvec", "attention", "o_proj_matvec", "gate_up_matvec", "down_matvec", "fused_decode_layer"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1280)
    ap.add_argument("--warmup", type=int, default=128)
    ap.add_argument("--sets", type=int, default=8, help="distinct weight sets rotated through")
    ap.add_argument("--mode", choices=["graph", "eager"], default="graph",
                    help="graph: the 64-call schedule is captured once in a HIP graph and replayed (Sec. 4.5 of the paper)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the CPU-oracle baseline leg (0 = skip)")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--path", choices=["fused", "stepwise"], default="stepwise",
                    help="fused: one persistent kernel per layer call (default); stepwise: the six-kernel path")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported" % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import workloads as wl
    from paper_2311_02103_amd import binding as rx
    from paper_2311_02103_amd.runtime import DeviceLayer, f16_bits, to_device

    rx.lib()
    rx.check(rx.relax_set_option("fused_decode", 1 if args.path == "fused" else 0))
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)
    shape, cap, seed, ncalls = wl.LLAMA7B, 4096, 1, 64

    # ---- inputs (all seeded, generated on the host, resident in HBM before the timed region) -------------------
    t_setup = time.time()
    Ls = [int(v) for v in wl.uniform_lengths(seed, ncalls, 1, cap)]
    kv_k, kv_v = wl.kv_prefill(shape, seed, 1, cap)
    host_w0 = None
    layers = []
    for s in range(args.sets):
        w = wl.layer_weights(shape, seed, layer=s)
        if s == 0:
            host_w0 = w
        lay = DeviceLayer(w, hidden=shape.hidden, n_heads=shape.n_heads, n_kv_heads=shape.n_kv_heads,
                          head_dim=shape.head_dim, ffn=shape.ffn, kv_capacity=cap, n_max=1, device=dev,
                          share_from=layers[0] if layers else None)
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

    graph = None
    if args.mode == "graph":
        with torch.cuda.stream(stream):
            run_eager(ncalls)                       # everything touched once before capture
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            run_eager(ncalls)

    def run(nsteps):
        if graph is None:
            run_eager(nsteps)
        else:
            full, rest = divmod(nsteps, ncalls)
            with torch.cuda.stream(stream):
                for _ in range(full):
                    graph.replay()
            run_eager(rest)

    # ---- timed region -------------------------------------------------------------------------------------------
    run(args.warmup)
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(args.steps)
    stream.synchronize()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    value = args.steps / elapsed

    mean_L = float(np.mean([Ls[i % ncalls] for i in range(args.steps)]))
    kvb = shape.kv_bytes_per_token()
    layer_bytes = shape.packed_bytes_per_layer() + kvb * mean_L + kvb + 6 * shape.hidden * 2
    layer_gbs = layer_bytes / (ms_per_step * 1e-3) / 1e9

    # ---- per-kernel timing of the same steps with HIP events on the launch stream (eager launches) --------------
    kernel_ms = {}
    kvb_call = lambda c: shape.packed_bytes_per_layer() + kvb * Ls[c] + kvb + 6 * shape.hidden * 2
    timed_bytes = {}
    if not args.no_kernel_timing:
        nk = min(args.steps, 256)
        step_ids = [5] if args.path == "fused" else [0, 1, 2, 3, 4]
        for step_id in step_ids:
            name = STEP_NAMES[step_id]
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(nk)]
            for a, b in evs:                        # materialise the hipEvent handles
                a.record(stream), b.record(stream)
            stream.synchronize()
            for i, (a, b) in enumerate(evs):
                rx.relax_profile_step_events(a.cuda_event, b.cuda_event, step_id)
                calls[i % ncalls](sh)
            stream.synchronize()
            kernel_ms[name] = float(np.mean([a.elapsed_time(b) for a, b in evs]))
            timed_bytes[name] = float(np.mean([kvb_call(i % ncalls) for i in range(nk)]))
    m, k = shape.matrices()["wgu"]
    gu_bytes = m * (k // 2) + m * (k // 32) * 2 + shape.hidden * 4 + shape.hidden * 2 + shape.ffn * 2
    roofline = None
    traffic = None
    if args.path == "fused" and "fused_decode_layer" in kernel_ms:
        tpath = os.path.join(ROOT, "profiles", "traffic_fused_decode_layer_7b.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
        nbytes, ms = timed_bytes["fused_decode_layer"], kernel_ms["fused_decode_layer"]
        ach = nbytes / (ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "decode_layer_kernel<128,1> (whole layer: 113.84 MB packed weights + 16 KB*L KV "
                                                "+ activations per launch)",
                    "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4),
                    "traffic": traffic, "algorithmic_bytes_per_launch": int(nbytes), "avg_launch_ms": round(ms, 5)}
    elif "gate_up_matvec" in kernel_ms:
        ach = gu_bytes / (kernel_ms["gate_up_matvec"] * 1e-3) / 1e9
        tpath = os.path.join(ROOT, "profiles", "traffic_gate_up_matvec_7b.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get("hbm_bytes_per_launch")
        roofline = {"bound": "hbm", "kernel": "gemv_q4_kernel<X_F32_NORM, EPI_SWIGLU, fast> (gate/up, m=22016, k=4096)",
                    "achieved": round(ach, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(ach / PEAK_HBM_GBS, 4),
                    "traffic": traffic, "algorithmic_bytes_per_launch": gu_bytes,
                    "avg_launch_ms": round(kernel_ms["gate_up_matvec"], 5)}

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same calls; doubles as a parity check --
    cpu = None
    if args.cpu_seconds > 0:
        import oracle
        mats = shape.matrices()
        ow = oracle.LayerWeights(*(oracle.QMat(host_w0[nm + ".q"], host_w0[nm + ".s"], *mats[nm])
                                   for nm in ("wqkv", "wo", "wgu", "wdown")), host_w0["norm_attn"], host_w0["norm_ffn"])
        od = oracle.Dims(shape.hidden, shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.rms_eps,
                         shape.rope_base, cap)
        Kf = wl.f16_bits_to_f32(kv_k).reshape(1, cap, shape.n_kv_heads, shape.head_dim)
        Vf = wl.f16_bits_to_f32(kv_v).reshape(1, cap, shape.n_kv_heads, shape.head_dim)
        sample = [c for c in range(ncalls) if c % args.sets == 0]
        layers[0].load_cache(kv_k, kv_v)            # both sides start from the seeded pre-fill and append in the same order
        torch.cuda.synchronize()
        done, t_cpu, worst = 0, 0.0, 0.0
        for c in sample:
            t1 = time.perf_counter()
            ref = oracle.decoder_layer(od, ow, xs_host[c], Kf, Vf, oracle.Seqs([1], [Ls[c]]))
            t_cpu += time.perf_counter() - t1
            done += 1
            calls[c](sh)
            stream.synchronize()
            got = f16_bits(outs[c]).view(np.float16).astype(np.float32)
            err = np.abs(got - ref)
            assert np.all(err <= 1e-2 + 2e-2 * np.abs(ref)), "bench: GPU output of call %d is outside tolerance" % c
            worst = max(worst, float(err.max()))
            if t_cpu > args.cpu_seconds and done >= 2:
                break
        cpu = {"value": round(done / t_cpu, 3), "unit": "tokens/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "%d of the 64 (n=1, L) calls (those on weight set 0), %.1f s of oracle time; GPU outputs of the "
                         "same calls checked against it, max abs err %.2e" % (done, t_cpu, worst)}

    line = {
        "metric": "decode tokens/s (7B-shaped int4, batch 1)", "value": round(value, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 (int4 weights, f32 accumulate)",
        "data": "synthetic",
        "config": {"workload": "configs[1]: one Llama-2-7B-shaped int4-g32 decoder layer, decode only, batch 1, n=1, "
                               "L~U{1..4096} over 64 seeded calls; 1 step = 1 token through 1 layer (a 32-layer model "
                               "does 32 such steps per token); %d rotating weight sets" % args.sets,
                   "mode": args.mode, "path": args.path, "mean_L": round(mean_L, 1), "build_id": rx.relax_build_id(),
                   "setup_s": round(setup_s, 1)},
        "layer_hbm": {"algorithmic_bytes_per_step": int(layer_bytes), "achieved_GBps": round(layer_gbs, 1),
                      "frac_of_peak": round(layer_gbs / PEAK_HBM_GBS, 4)},
        "kernel_ms": {k_: round(v, 5) for k_, v in kernel_ms.items()},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
