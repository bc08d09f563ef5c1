#!/usr/bin/env python3
"""Benchmark of the LQER W4A8 linear layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--cases headline|all]

A "step" is one pass of the whole hot path - quantize X to MXINT8, T = X_q A_k,
Y = X_q W_q + T B_k - over one batch of synthetic activations already resident in HBM.

The headline workload is the largest single-GPU configuration: the LLaMA-2-70B-shaped MLP layer
(W 8192 x 28672, k = 64) at M = 4096 tokens, the compute-bound regime of Sec. 2.1, priced against the
dense bf16 MFMA peak.  `cases` holds, first, the same layer at M = 16 and M = 1 (memory-bound regime,
priced against HBM bandwidth; consecutive steps walk a ring of distinct device copies whose packed
weights exceed the 256 MB last-level cache, so weights really come from HBM), then the 7B-shaped
decode and prefill layers, the stand-alone quantizer, the decode-to-prefill sweep of the 70B-shaped
layer, the seven linears of a 7B decoder block at 65536 tokens for k in {16, 32, 64}, and the offline
factor construction timed per layer.

Timed steps are enqueued as one HIP graph (captured once, replayed between two synchronisations):
decode steps last some tens of microseconds, less than a Python loop needs to launch them.  Kernel
durations come from events on the launch stream around graph replays of one stage alone.

Every roofline object prices a kernel against the vendor peak (`frac`) and against what the same chip
delivers for a kernel that does nothing else (`frac_measured`: a streaming read with the weight
kernel's access pattern, a register-resident MFMA loop; csrc/bench_probes.hip), and gives the fraction
the whole step reaches (`frac_step`).

Prints ONE JSON line.  `cpu_baseline` is the fp64 oracle timed on the host cores on a bounded sample
of the headline workload.
"""
from __future__ import annotations

import argparse
import ctypes as C
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
MFMA_INT8_PEAK_TOPS = 5000.0    # dense int8 MFMA, vendor figure
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


def bytes_prep_kernel(M, K, kp):
    """Algorithmic bytes of the projection kernel at prefill sizes: fp32 X in, bf16 X_q out, A_k once, T out."""
    return 4.0 * M * K + 2.0 * M * K + K * kp * 1.0625 + 4.0 * M * kp


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


# ---- peak probes ---------------------------------------------------------------------------------------------

_probes = None


def probes():
    """liblqer_probes.so (csrc/bench_probes.hip): kernels that only read, only copy, only issue MFMAs."""
    global _probes
    if _probes is None:
        import torch  # noqa: F401  (one HIP runtime for both libraries)
        path = os.path.join(ROOT, "paper_2402_02446_amd", "liblqer_probes.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2402_02446_amd.build`")
        L = C.CDLL(path)
        L.lqer_probe_stream_read.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.lqer_probe_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_void_p]
        L.lqer_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.lqer_probe_mfma_random.argtypes = [C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        L.lqer_probe_mfma_valu.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_void_p]
        _probes = L
    return _probes


def measure_peaks():
    """What this chip gives a kernel that does nothing else: HBM read and copy bandwidth on 1 GiB (four times the
    last-level cache), a read of 132 MB (the 70B-shaped layer's weight bytes, as a ring of five buffers so that
    each pass comes from HBM), and the 32x32x16 bf16 MFMA rate with one and with two wavefronts per SIMD."""
    import torch
    P = probes()
    cur = lambda: torch.cuda.current_stream().cuda_stream      # read per call: a graph capture runs on a stream of its own
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    big = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")          # 1 GiB
    dst = torch.empty_like(big)
    cus = torch.cuda.get_device_properties(0).multi_processor_count

    def chk(rc):
        if rc != 0:
            raise RuntimeError(f"probe launch failed: hip error {rc}")

    out = {}
    nbytes = big.numel() * 4
    best = (0.0, None)
    for wgs in (cus * 2, cus * 4, cus * 8, cus * 16):
        for fl in (4, 8, 16):
            f = lambda i: chk(P.lqer_probe_stream_read(big.data_ptr(), nbytes, sink.data_ptr(), wgs, fl, cur()))
            f(0)
            gbs = nbytes / (min(_event_ms(f, 4) for _ in range(2)) * 1e-3) / 1e9
            if gbs > best[0]:
                best = (gbs, (wgs, fl))
    out["hbm_read_gbs"] = best[0]
    out["hbm_read_best_launch"] = {"workgroups_of_256": best[1][0], "loads_of_1KiB_in_flight_per_wavefront": best[1][1]}
    f = lambda i: chk(P.lqer_probe_copy(big.data_ptr(), dst.data_ptr(), nbytes, cus * 8, cur()))
    f(0)
    ms = min(_event_ms(f, 5) for _ in range(3))
    out["hbm_copy_gbs"] = 2.0 * nbytes / (ms * 1e-3) / 1e9
    # the weight bytes of the 70B-shaped layer, ring of five distinct ranges of the 1 GiB buffer
    wbytes = int(8192 * 28672 * 0.5625) // 1024 * 1024
    wgs, fl = best[1]
    f = lambda i: chk(P.lqer_probe_stream_read(big.data_ptr() + (i % 5) * (200 << 20), wbytes, sink.data_ptr(), min(wgs, cus * 4), fl, cur()))
    for i in range(5):
        f(i)
    ms = min(_graph_ms(f, 20) for _ in range(2))
    out["hbm_read_132MB_us"] = ms * 1e3
    out["hbm_read_132MB_gbs"] = wbytes / (ms * 1e-3) / 1e9
    del big, dst
    for waves, key in ((1, "mfma_bf16_tflops_1wave_per_simd"), (2, "mfma_bf16_tflops_2waves_per_simd")):
        iters, chains = 4096, 8 if waves == 1 else 4
        wgs = cus * waves
        f = lambda i: chk(P.lqer_probe_mfma(wgs, iters, chains, sink.data_ptr(), cur()))
        f(0)
        ms = min(_event_ms(f, 3) for _ in range(3))
        out[key] = wgs * 4 * iters * chains * 32768.0 / (ms * 1e-3) / 1e12
    out["mfma_bf16_tflops"] = max(out["mfma_bf16_tflops_1wave_per_simd"], out["mfma_bf16_tflops_2waves_per_simd"])
    # the same loop on operands with random signs and significands: the data then toggles as in a real product, and the
    # chip's power management answers with a lower clock
    f = lambda i: chk(P.lqer_probe_mfma_random(cus * 2, 4096, 4, sink.data_ptr(), cur()))
    f(0)
    ms = min(_event_ms(f, 3) for _ in range(3))
    out["mfma_bf16_tflops_random_operands"] = cus * 2 * 4 * 4096 * 4 * 32768.0 / (ms * 1e-3) / 1e12
    # the matrix pipe beside vector work: two wavefronts per SIMD, n independent fp32 instructions behind every MFMA
    # (the tiled MXINT kernel has 2.7 per MFMA, the INT kernel 12: 8 of them the per-group conversion and scaling)
    beside = {}
    for int8, name, per in ((0, "bf16", 32768.0), (1, "int8", 65536.0)):
        for nv in (0, 4, 8, 12):
            iters, wgs = 4096, cus * 2
            f = lambda i: chk(P.lqer_probe_mfma_valu(wgs, iters, nv, int8, sink.data_ptr(), cur()))
            f(0)
            ms = min(_event_ms(f, 3) for _ in range(3))
            beside[f"{name}_{nv}_valu"] = wgs * 4 * iters * 4 * per / (ms * 1e-3) / 1e12
    out["mfma_beside_valu_tera_per_s"] = beside
    out["source"] = "csrc/bench_probes.hip, timed by events in this run"
    return out


def roofline(bound, kernel, work, ms_kernel, ms_step, work_step, peaks, traffic=None):
    """One roofline object: `work` algorithmic bytes (hbm) or flops (mfma) of the kernel per launch."""
    if bound == "hbm":
        ach, peak, unit = work / (ms_kernel * 1e-3) / 1e9, HBM_PEAK_GBS, "GB/s"
        meas = peaks.get("hbm_read_gbs") if peaks else None
        step = work_step / (ms_step * 1e-3) / 1e9 if ms_step else None
    else:
        ach, peak, unit = work / (ms_kernel * 1e-3) / 1e12, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s"
        meas = peaks.get("mfma_bf16_tflops") if peaks else None
        step = work_step / (ms_step * 1e-3) / 1e12 if ms_step else None
    r = {"bound": bound, "kernel": kernel, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
         "traffic": traffic}
    if meas:
        r["peak_measured"] = meas
        r["frac_measured"] = ach / meas
    rnd = peaks.get("mfma_bf16_tflops_random_operands") if (peaks and bound != "hbm") else None
    if rnd:
        # the MFMA loop alone on operands whose bits toggle like real data (the chip then clocks lower)
        r["peak_measured_random_operands"] = rnd
        r["frac_measured_random_operands"] = ach / rnd
    if step is not None:
        r["achieved_step"] = step
        r["frac_step"] = step / peak
    return r


def make_ring(rng, K, N, k, min_bytes):
    """A ring of distinct device copies of one layer (random canonical bytes) whose packed weights exceed
    min_bytes: what decides whether a step finds its weights in the last-level cache is their addresses."""
    from paper_2402_02446_amd import binding, synth
    per = K * N * 0.5625
    n = max(1, int(np.ceil(min_bytes / per)))
    d = synth.random_packed_layer(rng, K, N, k)
    layers = [binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"]) for _ in range(n)]
    return layers, d


def run_case(name, K, N, k, Ms, steps, warmup, rng, ring_bytes, gain, peaks):
    """Times the whole step and each kernel alone for every M in Ms on one ring of layers.
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
        if path == 1:
            res["roofline"] = roofline("hbm", "stream_kernel", bytes_main_kernel(M, K, N, kp), ms_main, ms_step,
                                       bytes_forward(M, K, N, kp), peaks)
        else:
            res["roofline"] = roofline("mfma", "tiled_kernel", fl, ms_main, ms_step, fl, peaks)
            if M >= 2048:
                res["roofline_prep_kernel"] = roofline("hbm", "prep_kernel", bytes_prep_kernel(M, K, kp), ms_prep, None, None, peaks)
        results.append(res)
        if ctx0 is None:
            # leave the result of layer 0 in Y for the oracle leg
            binding.lqer_linear_forward(layers[0], X, Y=Y)
            torch.cuda.synchronize()
            rows = min(M, 64)
            ctx0 = dict(packed=packed0, X=X_np[:rows], Y=Y[:rows].cpu().numpy(), M=M)
        del X, Y
    for l in layers:
        l.free()
    return results, ctx0


def run_quantizer_case(rows, cols, steps, rng, peaks):
    """lqer_quantize_mx alone on a cfg5-sized activation matrix: HBM-bound, 5.0625 B per element."""
    import torch
    from paper_2402_02446_amd import binding
    g = torch.Generator(device="cuda").manual_seed(int(rng.integers(1 << 31)))
    X = torch.randn((rows, cols), generator=g, device="cuda", dtype=torch.float32)
    f = lambda i: binding.lqer_quantize_mx(X, 8)
    f(0)
    torch.cuda.synchronize()
    ms = _event_ms(f, steps)
    r = roofline("hbm", "quantize_mx_kernel", rows * cols * 5.0625, ms, None, None, peaks)
    if peaks:
        # a quantizer reads 4 bytes and writes 1.0625 per element: the copy probe is the closer measured peak
        r["peak_measured"] = peaks["hbm_copy_gbs"]
        r["frac_measured"] = r["achieved"] / peaks["hbm_copy_gbs"]
    return {"workload": "a1 quantizer alone, %d x %d fp32 -> MXINT8" % (rows, cols), "M": rows, "K": cols,
            "ms_per_call": ms, "roofline": r}


def run_cfg5(steps, rng, peaks):
    """cfg5: the seven LQER linears of a LLaMA-7B decoder block at M = 32 x 2048 tokens, k in
    {16, 32, 64}; activations are drawn on the device (N(0,1), 1 % of channels x 50).  Returns one
    record per k with the per-shape times (whole step, projection kernel, main kernel) and the whole
    block's TFLOP/s, as seven separate calls and with one quantization per q/k/v and gate/up."""
    import torch
    from paper_2402_02446_amd import binding, synth
    M = synth.CFG5_M
    shapes = {}
    for name, K, N in synth.CFG5_LINEARS:
        shapes.setdefault((K, N), []).append(name)
    out = []
    g = torch.Generator(device="cuda").manual_seed(int(rng.integers(1 << 31)))
    Xs = {}
    for K in (4096, 11008):
        X = torch.randn((M, K), generator=g, device="cuda", dtype=torch.float32)
        ch = torch.from_numpy(synth.gen_outlier_channels(rng, K, max(1, round(0.01 * K)))).cuda()
        X[:, ch] *= 50.0
        Xs[K] = X
    med = lambda f, n: sorted(_event_ms(f, n) for _ in range(3))[1]
    for k in (16, 32, 64):
        total_ms, total_fl, per_shape, packed = 0.0, 0.0, [], {}
        for (K, N), names in shapes.items():
            d = synth.random_packed_layer(rng, K, N, k)
            packed[(K, N)] = d
            layer = binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"])
            X = Xs[K]
            Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
            f = lambda i: binding.lqer_linear_forward(layer, X, Y=Y)
            f_prep = lambda i: binding.lqer_linear_forward_ex(layer, X, Y=Y, stages=1)
            f_main = lambda i: binding.lqer_linear_forward_ex(layer, X, Y=Y, stages=2)
            f(0)
            torch.cuda.synchronize()
            ms, ms_prep, ms_main = med(f, steps), med(f_prep, steps), med(f_main, steps)
            fl = flops_forward(M, K, N, layer.kp)
            per_shape.append({"K": K, "N": N, "linears": names, "ms_per_linear": ms, "ms_prep_kernel": ms_prep,
                              "ms_main_kernel": ms_main, "tflops": fl / (ms * 1e-3) / 1e12,
                              "roofline": roofline("mfma", "tiled_kernel", fl, ms_main, ms, fl, peaks),
                              "roofline_prep_kernel": roofline("hbm", "prep_kernel", bytes_prep_kernel(M, K, layer.kp),
                                                               ms_prep, None, None, peaks)})
            total_ms += ms * len(names)
            total_fl += fl * len(names)
            layer.free()
            del Y
        # q/k/v and gate/up consume the same activations: one quantization per group (lqer_linear_forward_shared)
        shared, saved_ms = [], 0.0
        for names, K, N in ((("q", "k", "v"), 4096, 4096), (("gate", "up"), 4096, 11008)):
            d = packed[(K, N)]
            group = [binding.lqer_layer_import(K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"]) for _ in names]
            X = Xs[K]
            Ys = [torch.empty((M, N), dtype=torch.float32, device="cuda") for _ in names]
            ws = torch.empty(binding.lqer_linear_shared_workspace_bytes(group, M), dtype=torch.uint8, device="cuda")
            f_sh = lambda i: binding.lqer_linear_forward_shared(group, X, Ys=Ys, workspace=ws)
            f_sep = lambda i: [binding.lqer_linear_forward(l, X, Y=y, workspace=ws) for l, y in zip(group, Ys)]
            f_sh(0); f_sep(0)
            torch.cuda.synchronize()
            ms_sh, ms_sep = med(f_sh, steps), med(f_sep, steps)
            shared.append({"linears": list(names), "ms_shared": ms_sh, "ms_separate": ms_sep})
            saved_ms += ms_sep - ms_sh
            for l in group:
                l.free()
            del Ys, ws
        tf = total_fl / (total_ms * 1e-3) / 1e12
        tf_sh = total_fl / ((total_ms - saved_ms) * 1e-3) / 1e12
        out.append({"workload": "cfg5: LLaMA-7B decoder block, 7 LQER linears, M=%d" % M, "k": k,
                    "ms_per_block": total_ms, "tflops": tf, "frac_of_mfma_peak": tf / MFMA_BF16_PEAK_TFLOPS,
                    "per_shape": per_shape, "shared_activations": shared,
                    "ms_per_block_shared": total_ms - saved_ms, "tflops_shared": tf_sh,
                    "frac_of_mfma_peak_shared": tf_sh / MFMA_BF16_PEAK_TFLOPS})
    return out


def run_crossover(rng, peaks, steps=10):
    """cfg4: the 70B-shaped MLP layer swept over M = 1 .. 4096 to locate where the forward pass stops
    being bound by the weight stream (Sec. 2.1: memory-bound few-token regime against compute-bound
    prefill).  One layer (132 MB of weights, so successive steps may find part of it in the 256 MB
    last-level cache: this sweep compares M against M, it is not a bandwidth claim).  Each point gives the
    whole step against the roofline that binds at that M: max(bytes / 8 TB/s, flops / 2.5 PFLOP/s)."""
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
        f_main = lambda i: binding.lqer_linear_forward_ex(layer, X, Y=Y, stages=2)
        f(0)
        torch.cuda.synchronize()
        ms = _graph_ms(f, steps)
        ms_main = _graph_ms(f_main, steps)
        fl, by = flops_forward(M, K, N, layer.kp), bytes_forward(M, K, N, layer.kp)
        t_hbm, t_mfma = by / (HBM_PEAK_GBS * 1e9) * 1e3, fl / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e3
        out.append({"M": M, "path": "streaming" if binding.lqer_linear_path(layer, M) == 1 else "tiled",
                    "ms_per_step": ms, "ms_main_kernel": ms_main, "tflops": fl / (ms * 1e-3) / 1e12, "gbs": by / (ms * 1e-3) / 1e9,
                    "bound": "hbm" if t_hbm >= t_mfma else "mfma",
                    "frac_step_of_binding_roofline": max(t_hbm, t_mfma) / ms,
                    "frac_main_kernel_of_binding_roofline": max(t_hbm, t_mfma) / ms_main})
        del X, Y
    layer.free()
    # the ridge: smallest M whose step takes 1.5 x the M = 1 step or more
    base = out[0]["ms_per_step"]
    ridge = next((r["M"] for r in out if r["ms_per_step"] >= 1.5 * base), None)
    return {"workload": "cfg4: 8192 x 28672, k = 64, whole step", "sweep": out, "first_M_at_1p5x_of_M1": ridge,
            "ideal_ridge_M": 88}


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


def run_w2a8(rng, peaks):
    """The W2A8 setup (2-bit weight mantissas, rank 256: Sec. 4.1, Sec. 4.4) on the LLaMA-7B-shaped q_proj and MLP up
    layers: decode on a ring of device copies beyond the last-level cache, and prefill at M = 2048.  Bytes per weight
    of the packed W_q: 2 / 8 + 1 / 16 = 0.3125."""
    import torch
    from paper_2402_02446_amd import binding, synth
    out = []
    for (name, K, N, k) in (("W2A8 7B q_proj", 4096, 4096, 256), ("W2A8 7B MLP up", 4096, 11008, 256)):
        kp = k
        per = K * N * 0.3125
        d = synth.random_packed_layer(rng, K, N, k, w_bits=2)
        n = max(1, int(np.ceil(1.25 * LLC_BYTES / per)))
        layers = [binding.lqer_layer_import_w(2, K, N, k, d["Wc"], d["We"], d["Ac"], d["Ae"], d["Bc"], d["Be"]) for _ in range(n)]
        for M in (16, 2048):
            X = torch.randn((M, K), device="cuda", dtype=torch.float32)
            Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
            for l in layers:
                l.workspace(M)
            f = lambda i: binding.lqer_linear_forward(layers[i % n], X, Y=Y)
            f_main = lambda i: binding.lqer_linear_forward_ex(layers[i % n], X, Y=Y, stages=2)
            for i in range(n):
                f(i)
            torch.cuda.synchronize()
            steps = 2 * n if M <= 16 else 10
            ms, ms_main = _graph_ms(f, steps), _graph_ms(f_main, steps)
            fl = flops_forward(M, K, N, kp)
            by_main = K * N * 0.3125 + kp * N * 1.0625 + M * K * 1.0625 + 4.0 * M * kp + 4.0 * M * N
            by_step = K * N * 0.3125 + K * kp * 1.0625 + kp * N * 1.0625 + 4.0 * M * K + 4.0 * M * N
            path = binding.lqer_linear_path(layers[0], M)
            rec = {"workload": name, "M": M, "K": K, "N": N, "k": k, "w_bits": 2, "ring_layers": n,
                   "path": "streaming" if path == 1 else "tiled", "ms_per_step": ms, "ms_main_kernel": ms_main,
                   "tflops": fl / (ms * 1e-3) / 1e12}
            rec["roofline"] = (roofline("hbm", "stream_kernel", by_main, ms_main, ms, by_step, peaks) if path == 1
                               else roofline("mfma", "tiled_kernel", fl, ms_main, ms, fl, peaks))
            out.append(rec)
            del X, Y
        for l in layers:
            l.free()
    return out


def run_int_variant(rng, peaks):
    """The scaled-integer variant (Table 2 "L2QER-INT": INT4 g128 weights, INT8 per-token activations, k = 32) on the
    LLaMA-7B-shaped layers: decode on a ring of device copies beyond the last-level cache, prefill at M = 2048 and the
    4096 x 4096 linear at 65536 tokens.  One step = per-token quantizer + projection + main product (three launches; with
    few tokens both products split K over planes of workgroups and a small kernel adds the planes: five launches);
    the fractions are of the whole step: against HBM for M = 16 (0.515625 B per weight), against the dense int8
    matrix-core peak (5.0 POP/s) for prefill."""
    import torch
    from paper_2402_02446_amd import binding, synth
    out = []
    for (name, K, N, k, Ms) in (("INT 7B q_proj", 4096, 4096, 32, (16, 65536)), ("INT 7B MLP up", 4096, 11008, 32, (2048,)),
                                ("INT 7B MLP down", 11008, 4096, 32, (2048,))):
        d = synth.random_int_layer(rng, K, N, k)
        kp = d["kp"]
        per = K * N * 0.515625
        n = max(1, int(np.ceil(1.25 * LLC_BYTES / per))) if 16 in Ms else 1
        layers = [binding.lqer_int_layer_import(K, N, k, d["Wc"], d["Ws"], d["Ac"], d["As"], d["Bc"], d["Bs"]) for _ in range(n)]
        for M in Ms:
            X = torch.randn((M, K), device="cuda", dtype=torch.float32)
            Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
            for l in layers:
                l.workspace(M)
            f = lambda i: binding.lqer_linear_forward(layers[i % n], X, Y=Y)
            for i in range(n):
                f(i)
            torch.cuda.synchronize()
            steps = 2 * n if M <= 16 else (10 if M <= 2048 else 3)
            ms = _graph_ms(f, steps)
            ops = flops_forward(M, K, N, kp)
            by = K * N * 0.515625 + K * kp * 1.015625 + kp * N * 1.0 + 4.0 * M * K + 4.0 * M * N
            rec = {"workload": name, "M": M, "K": K, "N": N, "k": k, "format": "INT4 g128 / INT8 per token",
                   "ring_layers": n, "ms_per_step": ms, "tops": ops / (ms * 1e-3) / 1e12}
            if M <= 16:
                ach = by / (ms * 1e-3) / 1e9
                rec["roofline"] = {"bound": "hbm", "kernel": "whole step (quant_token_kernel + 2 x (int_gemm_kernel + int_reduce_planes_kernel))", "achieved": ach,
                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": None}
            else:
                ach = ops / (ms * 1e-3) / 1e12
                rec["roofline"] = {"bound": "mfma", "kernel": "whole step (quant_token_kernel + 2 x int_gemm_kernel)", "achieved": ach,
                                   "peak": MFMA_INT8_PEAK_TOPS, "unit": "TOP/s", "frac": ach / MFMA_INT8_PEAK_TOPS, "traffic": None}
                # what the int8 pipe delivers with this kernel's 12 vector instructions per MFMA beside it (probe)
                lim = (peaks or {}).get("mfma_beside_valu_tera_per_s", {}).get("int8_12_valu")
                if lim:
                    rec["roofline"]["peak_with_12_valu_per_mfma"] = lim
                    rec["roofline"]["frac_with_12_valu_per_mfma"] = ach / lim
            out.append(rec)
            del X, Y
        for l in layers:
            l.free()
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


def cpu_baseline(ctx, K, N, kp, budget_s=20.0):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the headline workload
    (its first rows: rows are independent, so the cost per row is the same for the rest, apart from the
    dequantization of the layer, which the oracle repeats per call), and the GPU result of those rows checked
    against it.  Only this function touches oracle/."""
    from oracle import factors, forward
    p = ctx["packed"]
    layer = factors.PackedLayer(K=p["K"], N=p["N"], k=p["k"], kp=p["kp"], Wc=p["Wc"], We=p["We"],
                                Ac=p["Ac"], Ae=p["Ae"], Bc=p["Bc"], Be=p["Be"])
    X = ctx["X"]
    rows = X.shape[0]
    t0 = time.perf_counter()
    Yref = forward.forward(X, layer)
    first = time.perf_counter() - t0
    reps, total = 1, first
    while total + first < budget_s and reps < 50:
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
    return {"value": flops_forward(rows, K, N, kp) / sec / 1e12, "unit": "TFLOP/s", "cores": cores,
            "kind": "oracle", "seconds_per_forward": sec,
            "sample": f"the first {rows} of the headline workload's {ctx['M']} token rows, all {N} output columns "
                      f"({K}x{N}, kp={kp}), whole oracle forward in fp64 numpy (layer dequantized per call), "
                      f"{reps} repetition(s); flops counted for those {rows} rows",
            "gpu_vs_oracle_rel_frobenius": err}


PMC_COPY_BYTES = 1 << 30


def pmc_probe(rng, which):
    """Workload for `rocprofv3 --pmc` runs.  Every probe starts with three plain copies of 1 GiB
    (copy_kernel of csrc/bench_probes.hip: reads and writes PMC_COPY_BYTES), which calibrate FETCH_SIZE /
    WRITE_SIZE in the same run.  `headline` / `cfg4_prefill`: the 70B-shaped layer at M = 4096;
    `cfg4_decode`: the same layer at M = 16 on a ring of device copies; `cfg2_decode`: the 7B-shaped
    q_proj at M = 16 on its ring; `cfg3`: the two 7B-shaped MLP layers at M = 2048; `cfg5_prep`: the 7B block's
    4096- and 11008-wide linears at M = 65536 (projection kernel and main kernel); `int_prefill`: the INT variant's
    three kernels on a 4096 x 4096 layer at 16384 tokens."""
    import torch
    from paper_2402_02446_amd import binding, synth
    if which == "build":
        print(json.dumps({"build_factors_seconds_per_layer": time_build_factors(rng)}))
        return
    src = torch.ones(PMC_COPY_BYTES // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        rc = probes().lqer_probe_copy(src.data_ptr(), dst.data_ptr(), PMC_COPY_BYTES, 2048, torch.cuda.current_stream().cuda_stream)
        assert rc == 0
    torch.cuda.synchronize()
    del src, dst
    plans = {
        "headline": [(4096, 8192, 28672, 64, 0, 6)], "cfg4_prefill": [(4096, 8192, 28672, 64, 0, 6)],
        "cfg4_decode": [(16, 8192, 28672, 64, 2.1 * LLC_BYTES, 5)],
        "cfg2_decode": [(16, 4096, 4096, 32, 1.25 * LLC_BYTES, 3)],
        "cfg3": [(2048, 4096, 11008, 32, 0, 10), (2048, 11008, 4096, 32, 0, 10)],
        "cfg5_prep": [(65536, 4096, 4096, 32, 0, 4), (65536, 11008, 4096, 32, 0, 4)],
    }
    if which == "int_prefill":
        # the scaled-integer variant: 4096 x 4096, k = 32 at 16384 tokens (quantizer, projection, main product)
        d = synth.random_int_layer(rng, 4096, 4096, 32)
        layer = binding.lqer_int_layer_import(4096, 4096, 32, d["Wc"], d["Ws"], d["Ac"], d["As"], d["Bc"], d["Bs"])
        X = torch.randn((16384, 4096), device="cuda", dtype=torch.float32)
        Y = torch.empty((16384, 4096), dtype=torch.float32, device="cuda")
        for _ in range(4):
            binding.lqer_linear_forward(layer, X, Y=Y)
        torch.cuda.synchronize()
        print("pmc-probe int_prefill done")
        return
    for (M, K, N, k, ring, reps) in plans[which]:
        layers, _ = make_ring(rng, K, N, k, ring)
        if M >= 65536:
            X = torch.randn((M, K), device="cuda", dtype=torch.float32)
        else:
            ch = synth.gen_outlier_channels(rng, K, max(1, round(0.01 * K)))
            X = torch.from_numpy(synth.gen_activations(rng, M, K, ch, 50.0)).cuda()
        Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        for rep in range(reps):
            for l in layers:
                binding.lqer_linear_forward(l, X, Y=Y)
        torch.cuda.synchronize()
        print("pmc-probe %s done: %d-layer ring x%d at M=%d, %dx%d" % (which, len(layers), reps, M, K, N))
        for l in layers:
            l.free()
        del X, Y


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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--cases", default="all", choices=["headline", "all"],
                    help="headline: the 70B-shaped layer at M = 4096 only; all (default): every workload")
    ap.add_argument("--pmc-probe", nargs="?", const="headline", default=None,
                    choices=["headline", "cfg4_decode", "cfg4_prefill", "cfg2_decode", "cfg3", "cfg5_prep", "int_prefill", "build"],
                    help="run one workload a few times and exit, for rocprofv3 runs (each after plain 1 GiB "
                         "copies that calibrate the byte counters; build: the offline step per layer shape "
                         "of cfg5, host and device path, timings printed as JSON)")
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

    t_start = time.perf_counter()
    peaks = measure_peaks()
    K, N, k, kp, M = 8192, 28672, 64, 64, 4096
    steps = max(1, args.steps)
    heads, ctx = run_case("cfg4: LLaMA-2-70B MLP, prefill", K, N, k, [M], steps, args.warmup, rng, 0, 50.0, peaks)
    head = heads[0]
    cases, extra = [], {}
    if args.cases == "all":
        dsteps = max(20, steps)
        plan = [
            ("cfg4: LLaMA-2-70B MLP, decode", 8192, 28672, 64, [16, 1], dsteps, 2.1 * LLC_BYTES),
            ("cfg2: LLaMA-7B q_proj decode", 4096, 4096, 32, [16, 1], 2 * dsteps, 1.25 * LLC_BYTES),
            ("cfg3: LLaMA-7B MLP up, prefill", 4096, 11008, 32, [2048], dsteps, 0),
            ("cfg3: LLaMA-7B MLP down, prefill", 11008, 4096, 32, [2048], dsteps, 0),
        ]
        for (nm, k_, n_, r_, ms_, st_, ring) in plan:
            res, _ = run_case(nm, k_, n_, r_, ms_, st_, min(args.warmup, st_), rng, ring, 50.0, peaks)
            cases.extend(res)
        cases.append(run_quantizer_case(32 * 2048, 4096, 10, rng, peaks))
        extra["crossover"] = run_crossover(rng, peaks)
        extra["cfg5"] = run_cfg5(3, rng, peaks)
        extra["added_rows"] = run_added_rows(rng)
        extra["w2a8_rank256"] = run_w2a8(rng, peaks)
        extra["int_variant"] = run_int_variant(rng, peaks)
        extra["build_factors_seconds_per_layer"] = time_build_factors(rng)
    t_gpu = time.perf_counter() - t_start
    cpu = cpu_baseline(ctx, K, N, kp)
    rf = dict(head["roofline"], traffic=read_pmc_traffic("tiled_kernel.cfg4_M4096"))
    out = {
        "metric": METRIC, "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1,
        "steps": steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "cfg4: LLaMA-2-70B-shaped MLP layer on one GPU, W 8192x28672 MXINT4, X 4096x8192 fp32 -> MXINT8, "
                               "k=64 MXINT8 factors, prefill (largest single-GPU configuration)",
                   "M": M, "K": K, "N": N, "k": k},
        "roofline": rf,
        "cpu_baseline": cpu,
        "measured_peaks": peaks,
        "headline_detail": head, "cases": cases,
        "seconds_gpu_part": t_gpu,
    }
    out.update(extra)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
