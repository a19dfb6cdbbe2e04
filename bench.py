#!/usr/bin/env python3
"""Benchmark: one decode step of the 32-layer Pythia-2.8B-shaped stack
(4096 cached positions, batch 1, fp16 weights/KV, fp32 accumulate) replayed
from one HIP graph on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--mode M] [--no-cpu]

Prints ONE JSON line.  A "step" is one replay of the whole stack.  Inputs are
the seeded synthetic tensors of synth/ (resident in HBM before timing starts).
The roofline entry divides the algorithmic bytes of one replay by its average
duration measured with HIP events on the launch stream; cpu_baseline times the
CPU oracle on a few layers of the same workload on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
PAPER_CONTEXT = {"paper_speedup_vs_hf": 1.34,
                 "paper_hw": "RTX 5090-class, Pythia-2.8B, 2048 decode tokens (context only)"}


def read_traffic_note():
    """HBM traffic per replay from the committed rocprofv3 --pmc summary, if any."""
    path = os.path.join(ROOT, "profiles", "stack_decode_pythia2.8b_s4096_hbm_traffic.txt")
    try:
        vals = {}
        for line in open(path):
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                vals[k.strip()] = float(v.split()[0])
        return vals["fetch_bytes_per_replay"] + vals["write_bytes_per_replay"]
    except Exception:
        return None


def cpu_baseline(shape, layers, kvs, x, S, n_layers_sample):
    """The oracle as it stands, timed on `n_layers_sample` layers of the workload."""
    import oracle
    orc = oracle.load("f64")
    Ks = [kvs[l][0][0].copy() for l in range(n_layers_sample)]
    Vs = [kvs[l][1][0].copy() for l in range(n_layers_sample)]
    x0 = orc.half_to_real(x[0])
    # repeat the sample until about 10 s of CPU work have been timed
    t0 = time.perf_counter()
    n_eval = 0
    while True:
        cur = x0
        for l in range(n_layers_sample):
            cur = orc.block_decode(shape, layers[l], Ks[l], Vs[l], S, cur)
        n_eval += n_layers_sample
        dt = time.perf_counter() - t0
        if dt >= 10.0:
            break
    cores = len(os.sched_getaffinity(0))
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    per_token_us = dt / n_eval * shape.n_layers * 1e6
    # the same on one thread (two blocks are enough to time it)
    single = None
    try:
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        n_before = gomp.omp_get_max_threads()
        gomp.omp_set_num_threads(1)
        t1 = time.perf_counter()
        cur = x0
        for l in range(min(2, n_layers_sample)):
            cur = orc.block_decode(shape, layers[l], Ks[l], Vs[l], S, cur)
        single = (time.perf_counter() - t1) / min(2, n_layers_sample) * shape.n_layers * 1e6
        gomp.omp_set_num_threads(n_before)
    except OSError:
        pass
    return {"value": per_token_us, "unit": "us/token", "cores": cores, "kind": "oracle",
            "single_thread_us_per_token": single,
            "sample": f"layers 0..{n_layers_sample - 1} of the same {shape.n_layers}-layer workload, "
                      f"{n_eval} block evaluations in {dt:.1f} s (fp64 C oracle, OpenMP over rows/heads), "
                      f"scaled to {shape.n_layers} layers per token",
            "seconds_measured": dt}


def bench_block(args):
    """The single-block workloads of the measurement table (not the headline):
    one block at batch 1, warm (one copy replayed) and cold (enough copies in
    rotation that their weights and caches exceed the 256 MB Infinity Cache), or
    one block at batch 8 with ragged lengths.  Prints one JSON line."""
    import numpy as np
    import torch
    import synth
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack

    shape = {"small": synth.SMALL_BLOCK, "2.8b": synth.PYTHIA_2_8B, "6.9b": synth.PYTHIA_6_9B}[args.shape]
    seed = synth.MASTER_SEED
    batch = args.batch
    if batch > 1:
        lens = synth.seq_lens(seed, batch, 1024, 8192)
        cap = int(lens.max()) + 1
    else:
        lens = np.array([args.ctx], dtype=np.int32)
        cap = args.ctx + 1
    L = args.layers
    ws = [synth.layer_weights(shape, seed, l) for l in range(L)]
    x = synth.x_input(shape, seed, batch)
    copies = []
    for _ in range(args.copies):
        ds = DeviceStack(shape, cap, batch, L)
        for l in range(L):
            ds.load_layer(l, ws[l])
            kv = synth.kv_cache(shape, seed, l, lens, cap, batch, poison=False)
            ds.load_kv(l, kv[0], kv[1], lens)
        ds.set_inputs(x, lens)
        ds.set_options(mode=args.mode, grid=args.grid, threads=args.threads)
        ds.capture()
        copies.append(ds)
    alg_bytes = cf.cfpp_algorithmic_bytes(copies[0].cfg, [int(v) for v in lens], L)
    footprint = args.copies * L * (cf.cfpp_packed_layer_bytes(copies[0].cfg) + cf.cfpp_kv_layer_bytes(copies[0].cfg))
    # every replay on ONE stream: the persistent kernels need the whole GPU to themselves
    one = copies[0].s
    for i in range(args.warmup):
        cf.cfpp_stack_replay(copies[i % args.copies].ctx, one)
    torch.cuda.synchronize()
    for ds in copies:
        ds.check()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        cf.cfpp_stack_replay(copies[i % args.copies].ctx, one)
    torch.cuda.synchronize()
    us = (time.perf_counter() - t0) / args.steps * 1e6
    for ds in copies:
        ds.check()
        ds.close()
    achieved = alg_bytes / (us * 1e-6) / 1e9
    print(json.dumps({
        "metric": f"us_per_step_decode_{L}L_{args.shape}_bs{batch}", "value": us, "unit": "us/step", "n_gpus": 1,
        "tokens_per_s": batch * 1e6 / us,
        "steps": args.steps, "warmup": args.warmup, "higher_is_better": False, "data": "synthetic",
        "dtype": "f16 weights/KV, f32 accumulate",
        "config": {"workload": f"{L} {shape.name} block(s), batch {batch}, cached positions {[int(v) for v in lens]}, "
                               f"{args.copies} cop{'y' if args.copies == 1 else 'ies'} replayed in rotation "
                               f"({footprint / 1e6:.0f} MB of weights and caches)",
                   "launch_mode": args.mode, "copies": args.copies},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "algorithmic_bytes_per_launch": alg_bytes},
    }))


def bench_prefill(args):
    """Prompt processing (cfpp_stack_prefill): a prompt of --tokens tokens through the whole stack from an
    empty cache, groups of 8 tokens per pass over the weights."""
    import numpy as np
    import torch
    import synth
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack

    shape = {"2.8b": synth.PYTHIA_2_8B, "6.9b": synth.PYTHIA_6_9B}[args.shape]
    seed, T, G = synth.MASTER_SEED, args.tokens, 8
    L = shape.n_layers
    ds = DeviceStack(shape, T + 1, G, L)
    for l in range(L):
        ds.load_layer(l, synth.layer_weights(shape, seed, l))
        kv = synth.kv_cache(shape, seed, l, 0, T + 1, G, poison=False)
        ds.load_kv(l, kv[0], kv[1], 0)
    ds.set_options(mode=0, grid=args.grid, threads=args.threads)
    xd = torch.from_numpy(synth.x_input(shape, seed, T)).to(ds.dev)
    od = torch.zeros_like(xd)
    torch.cuda.synchronize()
    run = lambda: cf.cfpp_stack_prefill(ds.ctx, ds.packed, ds.kv, xd, 0, T, 0, od, ds.s)
    for _ in range(args.warmup):
        run()
    ds.stream.synchronize()
    ds.check()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    ds.stream.synchronize()
    us = (time.perf_counter() - t0) / args.steps * 1e6
    ds.check()
    # what this path streams: per group of 8 tokens the weights once and every token's K/V rows
    streamed = sum(cf.cfpp_algorithmic_bytes(ds.cfg, list(range(t0_, min(t0_ + G, T))), L) for t0_ in range(0, T, G))
    h, f = shape.hidden, shape.ffn
    flops = 2.0 * (4 * h * h + 2 * h * f) * T * L + 4.0 * h * L * (T * (T + 1) / 2)
    ds.close()
    achieved = streamed / (us * 1e-6) / 1e9
    print(json.dumps({
        "metric": f"us_per_prompt_prefill_{L}L_{args.shape}_T{T}", "value": us, "unit": "us/prompt", "n_gpus": 1,
        "tokens_per_s": T * 1e6 / us, "steps": args.steps, "warmup": args.warmup, "higher_is_better": False,
        "data": "synthetic", "dtype": "f16 weights/KV, f32 accumulate",
        "config": {"workload": f"prompt of {T} tokens through {L} {shape.name} blocks from an empty cache, "
                               f"groups of {G} tokens (launch mode 0, batched projections)", "launch_mode": 0},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "streamed_bytes_per_prompt": streamed,
                     "note": "bytes this path streams: the weights once per group of 8 tokens; a prompt-sized "
                             "GEMM would read them once per prompt and be bound by the matrix cores instead"},
        "mfma": {"flops_per_prompt": flops, "achieved_TFLOPs": flops / (us * 1e-6) / 1e12,
                 "frac_of_f16_peak": flops / (us * 1e-6) / 2.5e15},
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--mode", type=int, default=int(os.environ.get("CFPP_MODE", "2")),
                    help="0: kernel per phase, 1: persistent per block, 2: persistent stack")
    ap.add_argument("--grid", type=int, default=int(os.environ.get("CFPP_GRID", "0")))
    ap.add_argument("--threads", type=int, default=int(os.environ.get("CFPP_THREADS", "512")))
    ap.add_argument("--ctx", type=int, default=4096, help="cached positions per layer")
    ap.add_argument("--workload", choices=["stack", "block", "prefill"], default="stack",
                    help="stack: the headline (32 layers, batch 1); block: one block, see --copies / --batch; "
                         "prefill: a prompt of --tokens tokens through the stack")
    ap.add_argument("--tokens", type=int, default=512, help="prefill workload: prompt length")
    ap.add_argument("--copies", type=int, default=1, help="block workload: copies replayed in rotation (cold when large)")
    ap.add_argument("--batch", type=int, default=1, help="block workload: sequences (ragged lengths 1024..8192 when > 1)")
    ap.add_argument("--layers", type=int, default=1, help="block workload: blocks in a row (a stack of that many layers)")
    ap.add_argument("--shape", choices=["small", "2.8b", "6.9b"], default="2.8b",
                    help="model shape of the stack (the headline metric is quoted on 2.8b, ctx 4096)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--gen-steps", type=int, default=64,
                    help="tokens of the generation-loop measurement reported beside the headline (0: skip)")
    ap.add_argument("--calibrate", action="store_true",
                    help="instead of the benchmark, run the plain copy kernel (1 GiB read + 1 GiB written per "
                         "launch, 5 launches) used to scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of it)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack

    if args.workload == "block":
        bench_block(args)
        return
    if args.workload == "prefill":
        if args.shape == "small":
            print("bench.py: the prefill workload runs at the 2.8b or 6.9b shape", file=sys.stderr)
            sys.exit(2)
        bench_prefill(args)
        return
    if args.shape == "small":
        print("bench.py: --shape small is a single-block workload (--workload block)", file=sys.stderr)
        sys.exit(2)
    if args.calibrate:
        n = 1 << 30
        src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        with cf.profile_build():                         # the calibration kernels live in the profiling build
            for _ in range(5):
                cf.cfpp_stream_copy(src, dst, n, 256, 512, None)
            torch.cuda.synchronize()
        print(json.dumps({"calibration": "cfpp_stream_copy", "bytes_read_per_launch": n,
                          "bytes_written_per_launch": n, "launches": 5}))
        return

    shape = synth.PYTHIA_2_8B if args.shape == "2.8b" else synth.PYTHIA_6_9B
    headline = args.shape == "2.8b" and args.ctx == 4096
    S, cap = args.ctx, args.ctx + 1 + (args.gen_steps + 8 if args.gen_steps > 0 else 0)
    seed = synth.MASTER_SEED
    t_gen = time.perf_counter()
    layers = synth.stack_weights(shape, seed, workers=16)
    ds = DeviceStack(shape, cap, 1)
    kvs = []
    for l in range(shape.n_layers):
        ds.load_layer(l, layers[l])
        kv = synth.kv_cache(shape, seed, l, S, cap, poison=False)
        ds.load_kv(l, kv[0], kv[1], S)
        kvs.append(kv if l < 4 else None)      # the CPU leg only needs a few layers
    x = synth.x_input(shape, seed)
    ds.set_inputs(x, S)
    ds.set_options(mode=args.mode, grid=args.grid, threads=args.threads)
    t_gen = time.perf_counter() - t_gen

    ds.capture()
    for _ in range(args.warmup):
        ds.replay()
    ds.check()

    # timed region: exactly K replays between two synchronisations; HIP events on
    # the launch stream bracket every replay for the per-launch duration
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in evs:
        a.record(ds.stream)
        ds.replay()
        b.record(ds.stream)
    ds.stream.synchronize()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ds.check()
    per = np.array([a.elapsed_time(b) for a, b in evs]) * 1e3        # us per replay
    us_wall = wall / args.steps * 1e6
    us_launch = float(per.mean())

    alg_bytes = cf.cfpp_algorithmic_bytes(ds.cfg, [S], shape.n_layers)
    achieved = alg_bytes / (us_launch * 1e-6) / 1e9
    grid = cf.cfpp_get_option(ds.ctx, cf.OPT_GRID)
    out = {
        "metric": f"us_per_token_decode_32L_pythia{args.shape}_bs1",
        "value": us_wall,
        "unit": "us/token",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": us_wall / 1e3,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 weights/KV, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": f"32-layer Pythia-{args.shape.upper()}-shaped decode step, ctx {S}, batch 1, one HIP graph replay",
                   "hidden": shape.hidden, "n_heads": shape.n_heads, "head_dim": shape.head_dim,
                   "ffn": shape.ffn, "n_layers": shape.n_layers, "ctx": S, "batch": 1,
                   "launch_mode": args.mode, "grid": grid, "threads": args.threads},
        "tokens_per_s": 1e6 / us_wall,
        "us_per_block": us_wall / shape.n_layers,
        "us_per_replay_events": {"mean": us_launch, "median": float(np.median(per)),
                                 "min": float(per.min()), "p95": float(np.percentile(per, 95))},
        "achieved_hbm_GBps": achieved,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic_note() if headline and args.mode == 2 else None,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "kernel": f"k_stack_fused<{shape.head_dim}> (the whole 32-layer step is one launch)" if args.mode == 2
                     else "all kernels of one graph replay",
                     "launch": "one graph replay of the 32-layer step"},
        "context": PAPER_CONTEXT,
        "input_generation_s": t_gen,
    }
    if args.gen_steps > 0:
        # the same stack inside a true generation loop: embedding row of the current
        # token -> stack -> final LayerNorm + LM head (50304 rows) + argmax; the position
        # advances on the device and every replay appends one row to the caches
        head = synth.lm_head(shape, seed)
        ds.load_lm(head, synth.embedding(shape, seed))
        ds.set_tokens([1] * (S + 1), S)
        ds.generate_capture()
        for _ in range(8):
            ds.replay()
        ds.check()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.gen_steps):
            ds.replay()
        ds.stream.synchronize()
        torch.cuda.synchronize()
        gen_us = (time.perf_counter() - t0) / args.gen_steps * 1e6
        ds.check()
        lm_bytes = 2 * synth.VOCAB * shape.hidden
        out["generation"] = {"us_per_token": gen_us, "tokens_per_s": 1e6 / gen_us, "steps": args.gen_steps,
                             "vocab": synth.VOCAB, "first_position": S + 8,
                             "achieved_hbm_GBps": (alg_bytes + lm_bytes) / (gen_us * 1e-6) / 1e9,
                             "what": "one graph replay per token: embedding row, the stack step, final LayerNorm, "
                                     "LM head and argmax; position advanced on the device"}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(shape, layers, kvs, x, S, 4)
    ds.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
