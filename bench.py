#!/usr/bin/env python3
"""Benchmark of the LQER W4A8 linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cases headline|all]

A "step" is one pass of the whole hot path - quantize X to MXINT8, T = X_q A_k,
Y = X_q W_q + T B_k - over one batch of synthetic activations already resident in HBM.
The headline workload is the LLaMA-7B-shaped q_proj decode (W 4096 x 4096, k = 32, M = 16); so
that weights really come from HBM and not from the 256 MB last-level cache, consecutive steps
walk a ring of distinct layers whose packed weights total more than that cache.

The timed steps are enqueued as one HIP graph (captured once, replayed between two
synchronisations): decode steps last some 15 microseconds, less than a Python loop needs to
launch them, so an eager loop would time the interpreter.  The eager figure is reported beside it.

Prints ONE JSON line.  `value` is TFLOP/s of the whole step; `roofline` prices the dominant
kernel (the weight-streaming main kernel) against HBM bandwidth with its duration measured by
events on the launch stream; `cpu_baseline` is the fp64 oracle timed on the host cores on a
bounded sample of the same workload; `cases` adds the prefill and 70B-shaped workloads, each
with its own roofline object.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "LQER W4A8 linear: TFLOP/s + % roofline (HBM GB/s M<=16, MFMA util M>=2048)"
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, vendor figure
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA, vendor figure
LLC_BYTES = 256 << 20


def flops_forward(M, K, N, kp):
    return 2.0 * M * K * N + 2.0 * M * K * kp + 2.0 * M * kp * N


def bytes_forward(M, K, N, kp):
    """Algorithmic HBM bytes of one forward: packed W_q, A_k, B_k once, fp32 X in, fp32 Y out."""
    return K * N * 0.5625 + K * kp * 1.0625 + kp * N * 1.0625 + 4.0 * M * K + 4.0 * M * N


def bytes_main_kernel(M, K, N, kp):
    """Algorithmic bytes of the main kernel alone: W_q and B_k once, X_q in its MXINT8 form and
    T (fp32) in, fp32 Y out."""
    return K * N * 0.5625 + kp * N * 1.0625 + M * K * 1.0625 + 4.0 * M * kp + 4.0 * M * N


def _event_ms(fn, iters):
    """Average duration of fn() in ms, timed by events on the current (launch) stream."""
    import torch
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for i in range(iters):
        fn(i)
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) / iters


def _graph_ms(fn, iters, reps=3):
    """Average duration of fn() in ms when `iters` calls are captured once into a HIP graph and the
    graph is replayed: the launches then cost no host time, so kernels of a few microseconds are
    timed by the GPU and not by the Python loop around them.  Events on the replay stream, best of
    `reps` replays.  fn must not allocate or synchronise."""
    import torch
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(iters):
            fn(i)
    g.replay()
    torch.cuda.synchronize()
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    best = float("inf")
    for _ in range(reps):
        start.record()
        g.replay()
        stop.record()
        stop.synchronize()
        best = min(best, start.elapsed_time(stop) / iters)
    del g
    return best


def make_ring(rng, K, N, k, min_bytes):
    """A ring of distinct layers (random canonical bytes) whose packed weights exceed min_bytes."""
    from paper_2402_02446_amd import binding, synth
    per = K * N * 0.5625
    n = max(1, int(np.ceil(min_bytes / per)))
    layers, packed0 = [], None
    for i in range(n):
        d = synth.random_packed_layer(rng, K, N, k)
        if packed0 is None:
            packed0 = d
        layers.append(binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"]))
    return layers, packed0


def run_case(name, K, N, k, Ms, steps, warmup, rng, ring_bytes, gain, bound):
    """Times the whole step and the main kernel alone for every M in Ms on one ring of layers.
    Returns (list of result dicts, context of the first M for the oracle leg)."""
    import torch
    from paper_2402_02446_amd import binding, synth
    layers, packed0 = make_ring(rng, K, N, k, ring_bytes)
    kp = layers[0].kp
    n = len(layers)
    ch = synth.gen_outlier_channels(rng, K, max(1, round(0.01 * K)))
    results, ctx0 = [], None
    for M in Ms:
        X_np = synth.gen_activations(rng, M, K, ch, gain)
        X = torch.from_numpy(X_np).cuda()
        Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        for l in layers:
            l.workspace(M)
        step = lambda i: binding.lqer_linear_forward(layers[i % n], X, Y=Y)
        main_only = lambda i: binding.lqer_linear_forward_ex(layers[i % n], X, Y=Y, stages=2)
        prep_only = lambda i: binding.lqer_linear_forward_ex(layers[i % n], X, Y=Y, stages=1)
        for i in range(max(warmup, n)):       # every ring member has a valid workspace afterwards
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        ms_step_eager = (time.perf_counter() - t0) * 1e3 / steps
        # the timed region proper: exactly `steps` steps, enqueued as one HIP graph, between two
        # synchronisations (wall clock); the event figures below use the same graphs
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(steps):
                step(i)
        g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        ms_step = (time.perf_counter() - t0) * 1e3 / steps
        del g
        ms_main = _graph_ms(main_only, steps)
        ms_prep = _graph_ms(prep_only, steps)
        ms_fwd_ev = _graph_ms(step, steps)
        path = binding.lqer_linear_path(layers[0], M)
        fl = flops_forward(M, K, N, kp)
        res = {
            "workload": name, "M": M, "K": K, "N": N, "k": k,
            "path": "streaming" if path == 1 else "tiled",
            "ring_layers": n, "steps": steps, "launch": "hip graph replay", "ms_per_step": ms_step,
            "ms_per_step_eager_python": ms_step_eager, "ms_step_events": ms_fwd_ev,
            "ms_main_kernel": ms_main, "ms_prep_kernel": ms_prep,
            "tflops": fl / (ms_step * 1e-3) / 1e12,
            "gbs_step": bytes_forward(M, K, N, kp) / (ms_step * 1e-3) / 1e9,
        }
        if bound == "hbm" or path == 1:
            ach = bytes_main_kernel(M, K, N, kp) / (ms_main * 1e-3) / 1e9
            res["roofline"] = {"bound": "hbm", "kernel": "stream_kernel", "achieved": ach,
                               "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                               "traffic": None}
        else:
            ach = fl / (ms_main * 1e-3) / 1e12
            res["roofline"] = {"bound": "mfma", "kernel": "tiled_kernel", "achieved": ach,
                               "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                               "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None}
        results.append(res)
        if ctx0 is None:
            # leave the result of layer 0 in Y for the oracle leg
            binding.lqer_linear_forward(layers[0], X, Y=Y)
            torch.cuda.synchronize()
            ctx0 = dict(packed=packed0, X=X_np, Y=Y.cpu().numpy())
        del X, Y
    for l in layers:
        l.free()
    return results, ctx0


def run_quantizer_case(rows, cols, steps, rng):
    """lqer_quantize_mx alone on a cfg5-sized activation matrix: HBM-bound, 5.0625 B per element."""
    import torch
    from paper_2402_02446_amd import binding
    g = torch.Generator(device="cuda").manual_seed(int(rng.integers(1 << 31)))
    X = torch.randn((rows, cols), generator=g, device="cuda", dtype=torch.float32)
    f = lambda i: binding.lqer_quantize_mx(X, 8)
    f(0)
    torch.cuda.synchronize()
    ms = _event_ms(f, steps)
    ach = rows * cols * 5.0625 / (ms * 1e-3) / 1e9
    return {"workload": "a1 quantizer alone, %d x %d fp32 -> MXINT8" % (rows, cols), "M": rows, "K": cols,
            "ms_per_call": ms,
            "roofline": {"bound": "hbm", "kernel": "quantize_mx_kernel", "achieved": ach, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None}}


def run_cfg5(steps, rng):
    """cfg5: the seven LQER linears of a LLaMA-7B decoder block at M = 32 x 2048 tokens, k in
    {16, 32, 64}; activations are drawn on the device (N(0,1), 1 % of channels x 50).  Returns one
    record per k with the per-shape times and the whole block's TFLOP/s."""
    import torch
    from paper_2402_02446_amd import binding, synth
    M = synth.CFG5_M
    shapes = {}
    for name, K, N in synth.CFG5_LINEARS:
        shapes.setdefault((K, N), []).append(name)
    out = []
    g = torch.Generator(device="cuda").manual_seed(int(rng.integers(1 << 31)))
    for k in (16, 32, 64):
        total_ms, total_fl, per_shape = 0.0, 0.0, []
        for (K, N), names in shapes.items():
            d = synth.random_packed_layer(rng, K, N, k)
            layer = binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"])
            X = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32)
            ch = torch.from_numpy(synth.gen_outlier_channels(rng, K, max(1, round(0.01 * K)))).cuda()
            X[:, ch] *= 50.0
            Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
            f = lambda i: binding.lqer_linear_forward(layer, X, Y=Y)
            f(0)
            torch.cuda.synchronize()
            ms = sorted(_event_ms(f, steps) for _ in range(3))[1]
            fl = flops_forward(M, K, N, layer.kp)
            per_shape.append({"K": K, "N": N, "linears": names, "ms_per_linear": ms,
                              "tflops": fl / (ms * 1e-3) / 1e12})
            total_ms += ms * len(names)
            total_fl += fl * len(names)
            layer.free()
            del X, Y
        # q/k/v and gate/up consume the same activations: one quantization per group (lqer_linear_forward_shared)
        shared, saved_ms = [], 0.0
        for names, K, N in ((("q", "k", "v"), 4096, 4096), (("gate", "up"), 4096, 11008)):
            group = []
            for _ in names:
                d = synth.random_packed_layer(rng, K, N, k)
                group.append(binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"]))
            X = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32)
            Ys = [torch.empty((M, N), dtype=torch.float32, device="cuda") for _ in names]
            ws = torch.empty(binding.lqer_linear_shared_workspace_bytes(group, M), dtype=torch.uint8, device="cuda")
            f_sh = lambda i: binding.lqer_linear_forward_shared(group, X, Ys=Ys, workspace=ws)
            f_sep = lambda i: [binding.lqer_linear_forward(l, X, Y=y, workspace=ws) for l, y in zip(group, Ys)]
            f_sh(0); f_sep(0)
            torch.cuda.synchronize()
            ms_sh = sorted(_event_ms(f_sh, steps) for _ in range(3))[1]
            ms_sep = sorted(_event_ms(f_sep, steps) for _ in range(3))[1]
            shared.append({"linears": list(names), "ms_shared": ms_sh, "ms_separate": ms_sep})
            saved_ms += ms_sep - ms_sh
            for l in group:
                l.free()
            del X, Ys, ws
        out.append({"workload": "cfg5: LLaMA-7B decoder block, 7 LQER linears, M=%d" % M, "k": k,
                    "ms_per_block": total_ms, "tflops": total_fl / (total_ms * 1e-3) / 1e12,
                    "frac_of_mfma_peak": total_fl / (total_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                    "per_shape": per_shape, "shared_activations": shared,
                    "ms_per_block_shared": total_ms - saved_ms,
                    "tflops_shared": total_fl / ((total_ms - saved_ms) * 1e-3) / 1e12})
    return out


def run_crossover(rng, steps=10):
    """cfg4: the 70B-shaped MLP layer swept over M = 1 .. 4096 to locate where the forward pass stops
    being bound by the weight stream (Sec. 2.1: memory-bound few-token regime against compute-bound
    prefill).  One layer (132 MB of weights, so successive steps may find part of it in the 256 MB
    last-level cache: this sweep compares M against M, it is not a bandwidth claim)."""
    import torch
    from paper_2402_02446_amd import binding, synth
    K, N, k = 8192, 28672, 64
    d = synth.random_packed_layer(rng, K, N, k)
    layer = binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"])
    out = []
    for M in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096):
        X = torch.randn((M, K), device="cuda", dtype=torch.float32)
        Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        f = lambda i: binding.lqer_linear_forward(layer, X, Y=Y)
        f(0)
        torch.cuda.synchronize()
        ms = _graph_ms(f, steps)
        out.append({"M": M, "path": "streaming" if binding.lqer_linear_path(layer, M) == 1 else "tiled",
                    "ms_per_step": ms, "tflops": flops_forward(M, K, N, layer.kp) / (ms * 1e-3) / 1e12,
                    "gbs": bytes_forward(M, K, N, layer.kp) / (ms * 1e-3) / 1e9})
        del X, Y
    layer.free()
    # the ridge: smallest M whose step takes 1.5 x the M = 1 step or more
    base = out[0]["ms_per_step"]
    ridge = next((r["M"] for r in out if r["ms_per_step"] >= 1.5 * base), None)
    return {"workload": "cfg4: 8192 x 28672, k = 64, whole step", "sweep": out, "first_M_at_1p5x_of_M1": ridge}


def run_added_rows(rng):
    """Whole-step times of the widened rows beside the plain forward pass, same layer and tokens: result
    leaving as MXINT8 from the epilogue (lqer_linear_forward_requant) and MXINT6 activations (W4A6)."""
    import torch
    from paper_2402_02446_amd import binding, synth
    out = []
    for (name, K, N, k, M) in (("cfg3 up", 4096, 11008, 32, 2048), ("cfg4", 8192, 28672, 64, 16), ("cfg4", 8192, 28672, 64, 4096)):
        d = synth.random_packed_layer(rng, K, N, k)
        layer = binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"])
        X = torch.randn((M, K), device="cuda", dtype=torch.float32)
        Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        f_plain = lambda i: binding.lqer_linear_forward_ex(layer, X, Y=Y)
        f_rq = lambda i: binding.lqer_linear_forward_requant(layer, X)
        f_plain(0); f_rq(0)
        torch.cuda.synchronize()
        rec = {"workload": name, "M": M, "K": K, "N": N, "k": k}
        rec["ms_fp32_output"] = sorted(_graph_ms(f_plain, 6) for _ in range(3))[1]
        rec["ms_mxint8_output"] = sorted(_graph_ms(f_rq, 6) for _ in range(3))[1]
        layer.set_activation_bits(6)
        f_plain(0)
        torch.cuda.synchronize()
        rec["ms_fp32_output_mxint6_activations"] = sorted(_graph_ms(f_plain, 6) for _ in range(3))[1]
        out.append(rec)
        layer.free()
        del X, Y
    return out


def time_build_factors(rng):
    """Wall time of the offline step per layer shape of cfg5: lqer_build_factors (host fp64 + upload, from host
    arrays) and lqer_build_factors_device (device kernels + small host steps, from device tensors; second call,
    so that one-time module loading is not counted)."""
    import torch
    from paper_2402_02446_amd import binding, synth
    res = []
    for (K, N) in ((4096, 4096), (4096, 11008), (11008, 4096)):
        W = synth.gen_weight(rng, K, N)
        ch = synth.gen_outlier_channels(rng, K, max(1, round(0.01 * K)))
        calib = np.stack([synth.gen_activations(rng, 128, K, ch, 50.0)])
        t0 = time.perf_counter()
        layer = binding.lqer_build_factors(W, calib, 32, 1)
        host_s = time.perf_counter() - t0
        layer.free()
        Wd, cd = torch.from_numpy(W).cuda(), torch.from_numpy(calib).cuda()
        dev_s = None
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            layer = binding.lqer_build_factors_device(Wd, cd, 32, 1)
            dev_s = time.perf_counter() - t0
            layer.free()
        res.append({"K": K, "N": N, "k": 32, "mode": "L2QER", "seconds": host_s, "seconds_device_path": dev_s})
    return res


def cpu_baseline(ctx, M, K, N, kp, budget_s=12.0):
    """The oracle as it stands, timed on this machine's host cores on the headline workload, and the
    GPU result checked against it.  Only this function touches oracle/."""
    from oracle import factors, forward
    p = ctx["packed"]
    layer = factors.PackedLayer(K=p["K"], N=p["N"], k=p["k"], kp=p["kp"], Wc=p["Wc"], We=p["We"],
                                Ac=p["Ac"], Ae=p["Ae"], Bc=p["Bc"], Be=p["Be"])
    X = ctx["X"]
    t0 = time.perf_counter()
    Yref = forward.forward(X, layer)
    first = time.perf_counter() - t0
    reps, total = 1, first
    while total < budget_s and reps < 50:
        t0 = time.perf_counter()
        forward.forward(X, layer)
        total += time.perf_counter() - t0
        reps += 1
    sec = total / reps
    err = forward.rel_frobenius(ctx["Y"], Yref)
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    try:
        from threadpoolctl import threadpool_info
        blas = [i.get("num_threads", 0) for i in threadpool_info() if i.get("user_api") == "blas"]
        if blas:
            cores = min(cores, max(blas))
    except Exception:
        pass
    return {"value": flops_forward(M, K, N, kp) / sec / 1e12, "unit": "TFLOP/s", "cores": cores,
            "kind": "oracle", "seconds_per_forward": sec,
            "sample": f"whole forward of the headline workload (M={M}, {K}x{N}, kp={kp}) in fp64 numpy, "
                      f"{reps} repetitions",
            "gpu_vs_oracle_rel_frobenius": err}


PMC_COPY_BYTES = 1 << 30


def pmc_probe(rng, which):
    """Workload for `rocprofv3 --pmc` runs.  `headline`: a plain copy of known size (the calibration of
    FETCH_SIZE / WRITE_SIZE) followed by the headline ring; `cfg4_decode` / `cfg4_prefill`: the
    70B-shaped layer at M = 16 / M = 4096 (ring of layers for the decode case), for the counters
    that show what the streaming and the tiled kernel wait for."""
    import torch
    from paper_2402_02446_amd import binding, synth
    if which == "build":
        print(json.dumps({"build_factors_seconds_per_layer": time_build_factors(rng)}))
        return
    if which == "headline":
        src = torch.ones(PMC_COPY_BYTES // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)          # one elementwise kernel: reads and writes PMC_COPY_BYTES
        torch.cuda.synchronize()
        M, K, N, k, ring, reps = 16, 4096, 4096, 32, 1.25 * LLC_BYTES, 3
    elif which == "cfg4_decode":
        M, K, N, k, ring, reps = 16, 8192, 28672, 64, 2.1 * LLC_BYTES, 5
    else:
        M, K, N, k, ring, reps = 4096, 8192, 28672, 64, 0, 6
    layers, _ = make_ring(rng, K, N, k, ring)
    ch = synth.gen_outlier_channels(rng, K, max(1, round(0.01 * K)))
    X = torch.from_numpy(synth.gen_activations(rng, M, K, ch, 50.0)).cuda()
    Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    for rep in range(reps):
        for l in layers:
            binding.lqer_linear_forward(l, X, Y=Y)
    torch.cuda.synchronize()
    print("pmc-probe %s done: %d-layer ring x%d at M=%d" % (which, len(layers), reps, M))


def read_pmc_traffic(kernel):
    """Bytes per launch of `kernel` from profiles/pmc_traffic.txt (lines `key value`), or None."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) == 2 and parts[0] == kernel + ".traffic_bytes_per_launch":
                    return float(parts[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--cases", default="all", choices=["headline", "all", "full"],
                    help="headline: cfg2 only; all: + cfg3, cfg4 and the quantizer; full: + cfg5 and build_factors timing")
    ap.add_argument("--pmc-probe", nargs="?", const="headline", default=None,
                    choices=["headline", "cfg4_decode", "cfg4_prefill", "build"],
                    help="run one workload a few times and exit, for rocprofv3 runs (headline: after a "
                         "plain 1 GiB copy that calibrates the byte counters; build: the offline step per "
                         "layer shape of cfg5, host and device path, timings printed as JSON)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (sharding the layer over "
              "several GPUs is a design note, not built)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    from paper_2402_02446_amd import binding
    binding.lib()                                     # fail loudly if the HIP library is missing
    rng = np.random.default_rng(0)

    if args.pmc_probe:
        pmc_probe(rng, args.pmc_probe)
        return

    M, K, N, k = 16, 4096, 4096, 32
    heads, ctx = run_case("cfg2: LLaMA-7B q_proj decode", K, N, k, [16, 1], args.steps, args.warmup, rng,
                          ring_bytes=1.25 * LLC_BYTES, gain=50.0, bound="hbm")
    head = heads[0]
    cases = heads[1:]
    extra = {}
    if args.cases in ("all", "full"):
        ksteps = max(10, args.steps // 10)
        plan = [
            ("cfg3: LLaMA-7B MLP up, prefill", 4096, 11008, 32, [2048], ksteps, 0, "mfma"),
            ("cfg3: LLaMA-7B MLP down, prefill", 11008, 4096, 32, [2048], ksteps, 0, "mfma"),
            ("cfg4: LLaMA-2-70B MLP", 8192, 28672, 64, [1, 16], ksteps * 2, 2.1 * LLC_BYTES, "hbm"),
            ("cfg4: LLaMA-2-70B MLP", 8192, 28672, 64, [4096], max(5, ksteps // 4), 0, "mfma"),
        ]
        for (nm, k_, n_, r_, ms_, st_, ring, bound) in plan:
            res, _ = run_case(nm, k_, n_, r_, ms_, st_, min(args.warmup, st_), rng, ring, 50.0, bound)
            cases.extend(res)
        cases.append(run_quantizer_case(32 * 2048, 4096, ksteps, rng))
    if args.cases == "full":
        extra["crossover"] = run_crossover(rng)
        extra["cfg5"] = run_cfg5(3, rng)
        extra["added_rows"] = run_added_rows(rng)
        extra["build_factors_seconds_per_layer"] = time_build_factors(rng)
    kp = 32
    cpu = cpu_baseline(ctx, M, K, N, kp)
    out = {
        "metric": METRIC, "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "cfg2: LLaMA-7B-shaped q_proj decode, W 4096x4096 MXINT4, X 16x4096 -> MXINT8, "
                               "k=32 MXINT8 factors, ring of %d distinct layers" % head["ring_layers"],
                   "M": M, "K": K, "N": N, "k": k},
        "roofline": dict(head["roofline"], traffic=read_pmc_traffic("stream_kernel.cfg2_M16")),
        "cpu_baseline": cpu,
        "headline_detail": head, "cases": cases,
    }
    out.update(extra)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
