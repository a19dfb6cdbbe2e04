#!/usr/bin/env python3
"""Benchmark: one decode step of the 32-layer Pythia-2.8B-shaped stack
(4096 cached positions, batch 1, fp16 weights/KV, fp32 accumulate) replayed
from one HIP graph on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--mode M] [--no-cpu] [--no-configs]

Prints ONE JSON line.  A "step" is one replay of the whole stack.  Inputs are
the seeded synthetic tensors of synth/ (resident in HBM before timing starts).
The roofline entry divides the algorithmic bytes of one replay by its average
duration measured with HIP events on the launch stream; cpu_baseline times the
CPU oracle on a few layers of the same workload on the host cores.  Beside the
headline the line carries, under "configs", the other workloads of the
measurement table (single blocks warm and cold, the 6.9B-shaped stack, the
batch of 8 sequences, the context sweep), each with its microseconds, GB/s of
algorithmic bytes and roofline fraction.
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


KERNEL_SOURCES = ("fused_kernel.hip", "decode_blocks.h", "attention_blocks.h", "attention_common.h", "device_utils.h",
                  "layout.h", "decode_params.h")


def kernel_sources_digest():
    """Digest of the sources the dominant kernel is compiled from: the committed counter summary
    names the digest it was measured with, so a summary older than the kernel is not passed on."""
    import hashlib
    m = hashlib.sha256()
    for n in KERNEL_SOURCES:
        m.update(open(os.path.join(ROOT, "paper_2604_23553_amd", "csrc", n), "rb").read())
    return m.hexdigest()[:16]


def read_traffic_note():
    """HBM traffic per replay from the committed rocprofv3 --pmc summary (counters cannot be read
    from inside this run): (bytes, note).  None when the summary was measured on other kernel sources."""
    path = os.path.join(ROOT, "profiles", "stack_decode_pythia2.8b_s4096_hbm_traffic.txt")
    try:
        vals = {}
        for line in open(path):
            if "=" in line and not line.lstrip().startswith("#"):
                k, v = line.split("=", 1)
                vals[k.strip()] = v.split()[0]
        if vals.get("kernel_sources_digest") != kernel_sources_digest():
            return None, "profiles/ summary is older than the kernel sources: not reported"
        return (float(vals["fetch_bytes_per_replay"]) + float(vals["write_bytes_per_replay"]),
                "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, " + os.path.relpath(path, ROOT))
    except Exception:
        return None, "no counter summary under profiles/"


def time_replays(ctxs, stream, steps, warmup):
    """Mean microseconds per graph replay: `ctxs` (captured contexts) replayed in rotation on one
    torch stream, HIP events around the whole timed batch."""
    import torch
    import paper_2604_23553_amd as cf
    n = len(ctxs)
    for i in range(warmup):
        cf.cfpp_stack_replay(ctxs[i % n], stream.cuda_stream)
    stream.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for i in range(steps):
        cf.cfpp_stack_replay(ctxs[i % n], stream.cuda_stream)
    b.record(stream)
    stream.synchronize()
    return a.elapsed_time(b) * 1e3 / steps


def entry(us, alg_bytes, **kw):
    gbs = alg_bytes / (us * 1e-6) / 1e9
    d = {"us": round(us, 2), "GBps": round(gbs, 1), "frac": round(gbs / HBM_PEAK_GBS, 4), "algorithmic_bytes": alg_bytes}
    d.update(kw)
    return d


def secondary_configs(ds, layers, x, args):
    """The other workloads of the measurement table, beside the headline: µs per step, GB/s of
    algorithmic bytes and the roofline fraction each (HIP events on the launch stream).
    ds: the resident 2.8B stack of the headline; layers: its numpy weights."""
    import numpy as np
    import torch
    import synth
    import synth.device as sdev
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack
    seed = synth.MASTER_SEED
    out = {}
    MODE_NAMES = {-1: "auto", 0: "0 (phase kernels)", 1: "1", 2: "2 (whole-stack kernel)"}

    # context sweep of the 32-layer 2.8B stack (the paper's latency tables sweep 16 -> 2048
    # positions, Sec. 3 and appendix), default launch mode
    shape = ds.shape
    sweep = {}
    for S in (16, 128, 512, 1024, 2048, 4096):
        if S + 1 > ds.max_seq:
            continue
        ds.set_inputs(x, S)
        ds.capture()
        us = time_replays([ds.ctx], ds.stream, 40, 8)
        ds.check()
        sweep[str(S)] = entry(us, cf.cfpp_algorithmic_bytes(ds.cfg, [S], shape.n_layers))
    big = DeviceStack(shape, 8193, 1, share_weights_of=ds)         # same weights, a cache of 8192 positions
    for l in range(shape.n_layers):
        sdev.fill_kv(big.kv[l], seed, l)
    big.set_options(mode=args.mode, grid=args.grid, threads=args.threads)
    big.set_inputs(x, 8192)
    big.capture()
    us = time_replays([big.ctx], big.stream, 40, 8)
    big.check()
    sweep["8192"] = entry(us, cf.cfpp_algorithmic_bytes(big.cfg, [8192], shape.n_layers),
                          note="cache filled by the device generator (synth/device.py)")
    big.close()
    out["context_sweep_pythia2.8b_32L"] = {"unit": "us per token", "launch_mode": MODE_NAMES[args.mode], "by_cached_positions": sweep}

    def block_copies(shape_, lens, cap, batch, n_copies, w_np=None):
        cs = []
        for i in range(n_copies):
            c = DeviceStack(shape_, cap, batch, 1)
            if w_np is not None:
                c.load_layer(0, w_np)
            else:
                c.load_layer_device(0, sdev.layer_tensors(shape_, seed, 0, c.dev))
            sdev.fill_kv(c.kv[0], seed, i)
            c.set_inputs(synth.x_input(shape_, seed, batch), lens)
            cs.append(c)
        return cs

    def block_times(cs, lens, shape_, modes, steps):
        r = {}
        alg = cf.cfpp_algorithmic_bytes(cs[0].cfg, [int(v) for v in np.atleast_1d(lens)], 1)
        for mode in modes:
            try:
                for c in cs:
                    c.set_options(mode=mode)
                    c.capture()
                warm = time_replays([cs[0].ctx], cs[0].stream, steps, 20)
                cold = time_replays([c.ctx for c in cs], cs[0].stream, steps, 20) if len(cs) > 1 else None
                for c in cs:
                    c.check()
                r[MODE_NAMES[mode]] = {"warm": entry(warm, alg), "cold": entry(cold, alg) if cold else None}
            except cf.CfppError as e:
                r[MODE_NAMES[mode]] = {"error": str(e)}
        return r

    # config 1: the h-512 block, 128 cached positions; cold = 100 copies in rotation (> 600 MB)
    cs = block_copies(synth.SMALL_BLOCK, 128, 129, 1, 100, synth.layer_weights(synth.SMALL_BLOCK, seed, 0))
    out["cfg1_block_h512_s128"] = {"workload": "one h-512 block, 128 cached positions, batch 1 (6.6 MB: latency-bound; cold = 100 copies "
                                               "replayed in rotation)", "by_launch_mode": block_times(cs, 128, synth.SMALL_BLOCK, (-1, 0, 2), 300)}
    for c in cs:
        c.close()
    # config 2: one 2.8B-shaped block, 1024 cached positions; cold = 4 copies in rotation (672 MB > the 256 MB Infinity Cache)
    cs = block_copies(shape, 1024, 1025, 1, 4, layers[0])
    out["cfg2_block_pythia2.8b_s1024"] = {"workload": "one Pythia-2.8B-shaped block, 1024 cached positions, batch 1 (168 MB; cold = 4 copies "
                                                      "replayed in rotation, 70 % of the roofline = 29.97 us)",
                                          "by_launch_mode": block_times(cs, 1024, shape, (-1, 0, 2), 200)}
    for c in cs:
        c.close()
    # config 4: the 32-layer 6.9B-shaped stack, 2048 cached positions (weights from the device generator)
    s69 = synth.PYTHIA_6_9B
    d4 = DeviceStack(s69, 4097, 1)
    for l in range(s69.n_layers):
        d4.load_layer_device(l, sdev.layer_tensors(s69, seed, l, d4.dev))
        sdev.fill_kv(d4.kv[l], seed, l)
    d4.set_options(mode=args.mode, grid=args.grid, threads=args.threads)
    x69 = synth.x_input(s69, seed)
    d4.set_inputs(x69, 2048)
    d4.capture()
    us = time_replays([d4.ctx], d4.stream, 30, 6)
    d4.check()
    out["cfg4_stack_pythia6.9b_32L_s2048"] = entry(us, cf.cfpp_algorithmic_bytes(d4.cfg, [2048], s69.n_layers),
                                                   workload="32-layer Pythia-6.9B-shaped decode step, 2048 cached positions, batch 1, one graph replay",
                                                   launch_mode=MODE_NAMES[args.mode], tokens_per_s=round(1e6 / us, 1))
    # the same resident stack over the paper's context sweep (Sec. 3 and appendix: 16 -> 2048 positions), and 4096
    sweep69 = {}
    for S in (16, 128, 512, 1024, 2048, 4096):
        d4.set_inputs(x69, S)
        d4.capture()
        us = time_replays([d4.ctx], d4.stream, 20, 4)
        d4.check()
        sweep69[str(S)] = entry(us, cf.cfpp_algorithmic_bytes(d4.cfg, [S], s69.n_layers))
    out["context_sweep_pythia6.9b_32L"] = {"unit": "us per token", "launch_mode": MODE_NAMES[args.mode], "by_cached_positions": sweep69,
                                           "note": "weights and cache from the device generator (synth/device.py)"}
    d4.close()
    # config 5: one 6.9B-shaped block, 8 sequences with cached lengths drawn from [1024, 8192]
    lens = synth.seq_lens(seed, 8, 1024, 8192)
    cs = block_copies(s69, lens, int(lens.max()) + 1, 8, 1)
    r = block_times(cs, lens, s69, (-1,), 100)
    alg5 = cf.cfpp_algorithmic_bytes(cs[0].cfg, [int(v) for v in lens], 1)
    out["cfg5_block_pythia6.9b_batch8"] = {"workload": f"one Pythia-6.9B-shaped block, batch 8, cached positions {[int(v) for v in lens]} "
                                                       f"({alg5 / 1e9:.2f} GB per step: cold by construction; 70 % of the roofline = "
                                                       f"{alg5 / (0.7 * HBM_PEAK_GBS * 1e3):.0f} us)",
                                           "by_launch_mode": {k: v["warm"] if "warm" in v else v for k, v in r.items()}}
    cs[0].close()
    # prompt processing through the prompt-sized kernels: 512 tokens into the (now no longer needed) first
    # rows of the headline stack's caches, one pass
    T = 512
    if T < ds.max_seq:
        nbytes = cf.cfpp_prefill_scratch_bytes(ds.cfg, T)
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=ds.dev)
        xd = torch.from_numpy(synth.x_input(shape, seed, T)).to(ds.dev)
        od = torch.zeros_like(xd)
        run = lambda: cf.cfpp_stack_prefill_gemm(ds.ctx, ds.packed, ds.kv, xd, 0, T, 0, od, scratch, nbytes, T, ds.s)
        for _ in range(2):
            run()
        ds.stream.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(ds.stream)
        for _ in range(5):
            run()
        b.record(ds.stream)
        ds.stream.synchronize()
        ds.check()
        us = a.elapsed_time(b) * 1e3 / 5
        h, f, L = shape.hidden, shape.ffn, shape.n_layers
        flops = 2.0 * (4 * h * h + 2 * h * f) * T * L + 4.0 * h * L * (T * (T + 1) / 2)
        out["prefill_pythia2.8b_32L_T512"] = {
            "workload": "prompt of 512 tokens through the 32-layer stack from position 0, one pass (cfpp_stack_prefill_gemm)",
            "us": round(us, 1), "tokens_per_s": round(T * 1e6 / us, 1), "useful_TFLOPs": round(flops / us / 1e6, 1),
            "frac_of_f16_mfma_peak": round(flops / us / 1e6 / 2500.0, 4),
            "note": "the path through the batched projections (8 tokens per pass): python bench.py --workload prefill --gemm-rows 0"}
    return out


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
    """Prompt processing: a prompt of --tokens tokens through the whole stack from an empty cache.
    --gemm-rows 0: cfpp_stack_prefill (groups of 8 tokens per pass over the weights, batched projections);
    --gemm-rows N: cfpp_stack_prefill_gemm (N tokens per pass, GEMMs on the matrix cores)."""
    import numpy as np
    import torch
    import synth
    import paper_2604_23553_amd as cf
    from paper_2604_23553_amd.harness import DeviceStack

    shape = {"2.8b": synth.PYTHIA_2_8B, "6.9b": synth.PYTHIA_6_9B}[args.shape]
    seed, T = synth.MASTER_SEED, args.tokens
    rows = args.gemm_rows
    G = rows if rows else 8
    L = shape.n_layers
    ds = DeviceStack(shape, T + 1, 1 if rows else 8, L)
    for l in range(L):
        ds.load_layer(l, synth.layer_weights(shape, seed, l))
        kv = synth.kv_cache(shape, seed, l, 0, T + 1, 1 if rows else 8, poison=False)
        ds.load_kv(l, kv[0], kv[1], 0)
    ds.set_options(mode=0, grid=args.grid, threads=args.threads)
    xd = torch.from_numpy(synth.x_input(shape, seed, T)).to(ds.dev)
    od = torch.zeros_like(xd)
    if rows:
        nbytes = cf.cfpp_prefill_scratch_bytes(ds.cfg, rows)
        if nbytes == 0:
            raise SystemExit(f"--gemm-rows {rows}: a multiple of 128 up to 4096 is needed")
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=ds.dev)
        run = lambda: cf.cfpp_stack_prefill_gemm(ds.ctx, ds.packed, ds.kv, xd, 0, T, 0, od, scratch, nbytes, rows, ds.s)
    else:
        run = lambda: cf.cfpp_stack_prefill(ds.ctx, ds.packed, ds.kv, xd, 0, T, 0, od, ds.s)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        run()
    ds.stream.synchronize()
    ds.check()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(ds.stream)
    for _ in range(args.steps):
        run()
    b.record(ds.stream)
    ds.stream.synchronize()
    us = a.elapsed_time(b) * 1e3 / args.steps
    ds.check()
    # what the path streams: per pass of G tokens the weights once and every token's K/V rows
    streamed = sum(cf.cfpp_algorithmic_bytes(ds.cfg, [t0_], L) for t0_ in range(0, T, G))
    h, f = shape.hidden, shape.ffn
    flops = 2.0 * (4 * h * h + 2 * h * f) * T * L + 4.0 * h * L * (T * (T + 1) / 2)
    ds.close()
    achieved = streamed / (us * 1e-6) / 1e9
    tf = flops / (us * 1e-6) / 1e12
    line = {
        "metric": f"us_per_prompt_prefill_{L}L_{args.shape}_T{T}", "value": us, "unit": "us/prompt", "n_gpus": 1,
        "tokens_per_s": T * 1e6 / us, "steps": args.steps, "warmup": args.warmup, "higher_is_better": False,
        "data": "synthetic", "dtype": "f16 weights/KV, f32 accumulate",
        "config": {"workload": f"prompt of {T} tokens through {L} {shape.name} blocks from an empty cache, "
                               + (f"{rows} tokens per pass (GEMMs on the matrix cores, activations as fp16 head + remainder)" if rows
                                  else "groups of 8 tokens (batched projections)"), "tokens_per_pass": G},
        "mfma": {"flops_per_prompt": flops, "achieved_TFLOPs": tf, "frac_of_f16_peak": tf / 2500.0,
                 "note": "useful flops (2 per weight and token, 4 per attention pair and dimension); the GEMM path "
                         "issues twice as many in the projections (head and remainder of every activation)"},
        "hbm": {"streamed_bytes_per_prompt": streamed, "GBps": achieved, "frac": achieved / HBM_PEAK_GBS},
    }
    line["roofline"] = ({"bound": "mfma", "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0, "traffic": None}
                        if rows else
                        {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBS, "traffic": None})
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--mode", type=int, default=-1,
                    help="-1: automatic (the library's default), 0: kernel per phase, 1: persistent per block, "
                         "2: whole-stack kernel")
    ap.add_argument("--grid", type=int, default=0)
    ap.add_argument("--threads", type=int, default=512)
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the other workloads of the measurement table (reported under \"configs\")")
    ap.add_argument("--ctx", type=int, default=4096, help="cached positions per layer")
    ap.add_argument("--workload", choices=["stack", "block", "prefill"], default="stack",
                    help="stack: the headline (32 layers, batch 1); block: one block, see --copies / --batch; "
                         "prefill: a prompt of --tokens tokens through the stack")
    ap.add_argument("--tokens", type=int, default=512, help="prefill workload: prompt length")
    ap.add_argument("--gemm-rows", type=int, default=512,
                    help="prefill workload: tokens per pass of the prompt-sized kernels (a multiple of 128); 0 = the "
                         "batched path, 8 tokens per pass")
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
    fused = args.mode in (-1, 2)             # (the automatic mode runs a stack step in the whole-stack kernel)
    traffic, traffic_note = read_traffic_note() if headline and fused and args.grid == 0 and args.threads == 512 else (None, "not the profiled launch")
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
                   "launch_mode": "auto (whole-stack kernel)" if args.mode == -1 else args.mode, "grid": grid, "threads": args.threads},
        "tokens_per_s": 1e6 / us_wall,
        "us_per_block": us_wall / shape.n_layers,
        "us_per_replay_events": {"mean": us_launch, "median": float(np.median(per)),
                                 "min": float(per.min()), "p95": float(np.percentile(per, 95))},
        "achieved_hbm_GBps": achieved,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_note,
                     "algorithmic_bytes_per_launch": alg_bytes,
                     "kernel": f"k_stack_fused<{shape.head_dim}> (the whole 32-layer step is one launch)" if fused
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
    if headline and not args.no_configs:
        out["configs"] = secondary_configs(ds, layers, x, args)
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(shape, layers, kvs, x, S, 4)
    ds.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
