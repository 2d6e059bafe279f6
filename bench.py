#!/usr/bin/env python3
"""Benchmark of the per-bucket quantization hot path on one MI355X.

A step is one pass of the whole path over one synthetic gradient that is already resident in HBM:
ogq_quantize (statistics, level solve, encode, bit-pack) followed by ogq_dequantize_average of
the packed stream(s).  The default workload is the ResNet-50-sized BinGrad-b configuration
(25.6 M fp32, bucket 2048); --workload picks another one.  Inputs rotate over several distinct
buffers (>= 1 GB in total) so that the 256 MB last-level cache cannot serve repeats.

Prints ONE JSON line.  `value` is the fp32-gradient throughput of the whole step (4*n*workers
bytes per step / time per step); `roofline` prices the dominant kernel's algorithmic bytes per
launch against the HBM peak using HIP-event timings taken inside the timed region (the decoder's entry also
carries `cold_*` figures: the same kernel over packed streams that no cache holds);
`cpu_baseline` is the plain CPU oracle timed on the host cores, with OpenMP over buckets and on one
thread (a reported baseline only).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
WORKLOAD_NAMES = ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "pb2", "orq5", "orq3clip", "cfg2clip", "bin512", "sign2",
                  "tern3", "linear5", "orq3d32k", "orq3d128")


def algorithmic_bytes(n: int, bucket_size: int, bits: int, workers: int, levels_per_bucket: int):
    """Bytes the method must move per launch: quantize reads the gradient once and writes codes and
    levels; decode-average reads every worker's codes and levels and writes the fp32 average."""
    nb = (n + bucket_size - 1) // bucket_size
    codes = ((n + 63) // 64) * bits * 8
    levels = nb * levels_per_bucket * 4
    return 4 * n + codes + levels, workers * (codes + levels) + 4 * n


def read_traffic_note(kernel_key: str):
    """Measured HBM bytes per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy
    kernel of known size) as recorded in profiles/hbm_traffic.txt, or None."""
    return read_note("hbm_traffic.txt", kernel_key)


def read_note(file_name: str, kernel_key: str):
    """A figure recorded from a separate rocprofv3 counter run: `<workload>:<kernel> <value>` lines."""
    path = os.path.join(ROOT, "profiles", file_name)
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == kernel_key:
            try:
                return float(parts[1])
            except ValueError:
                return None
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2", choices=sorted(WORKLOAD_NAMES))
    ap.add_argument("--buffers", type=int, default=0, help="distinct input buffers (0 = enough for 1 GB)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--graph", action="store_true",
                    help="capture the K timed steps into one HIP graph and time its replay (same kernels, same order)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (simulated workers are buffers on that device); "
              "--gpus N with N > 1 is not supported.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import paper_2002_11082_amd as ogq
    from paper_2002_11082_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    ogq.lib()  # fail loudly if the HIP library is missing
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl = synth.WORKLOADS[args.workload]
    n, d, bits, W = wl.n, wl.bucket_size, wl.bits, wl.workers
    grad_bytes = 4 * n * W
    n_buf = args.buffers or max(2, -(-(1 << 30) // grad_bytes) + 1)
    if args.workload == "cfg2":
        n_buf = max(n_buf, 10)

    # ---- synthetic inputs, resident in HBM before anything is timed ------------------------------
    # Buffer 0 is the workload's own seeded gradient(s); the others hold the same values rolled by a
    # different amount (same distribution, different bytes at every address).
    host = [wl.gradient(w) for w in range(W)]
    grads = []  # grads[b][w]
    for b in range(n_buf):
        grads.append([torch.from_numpy(np.roll(h, 7919 * b) if b else h).to(dev) for h in host])
    params = [ogq.make_params(d, bits, wl.scheme, wl.level_iters, wl.philox_seed(w), 0, wl.clip_factor) for w in range(W)]
    n_levels = ogq.ogq_levels_count(n, params[0])
    n_words = ogq.ogq_codes_bytes(n, params[0]) // 8
    levels = [[torch.empty(n_levels + 4, dtype=torch.float32, device=dev) for _ in range(W)] for _ in range(n_buf)]
    codes = [[torch.empty(n_words + 2, dtype=torch.int64, device=dev) for _ in range(W)] for _ in range(n_buf)]
    outs = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(n_buf)]
    dparams = ogq.make_params(d, bits, wl.scheme)

    # Launch path of the timed loop: the raw C-ABI entry points with every argument marshalled ahead of
    # time, so that the host enqueues faster than the GPU drains and the HIP events that bracket each
    # kernel on this stream see back-to-back execution.
    import ctypes
    L = ogq.lib()
    stream = torch.cuda.Stream(dev)  # a real (non-null) stream, default priority
    torch.cuda.set_stream(stream)
    sp = ctypes.c_void_p(stream.cuda_stream)
    q_args, a_args, keep = [], [], []
    for b in range(n_buf):
        q_args.append([(ctypes.c_void_p(grads[b][w].data_ptr()), ctypes.c_size_t(n), ctypes.byref(params[w]),
                        ctypes.c_void_p(levels[b][w].data_ptr()), ctypes.c_void_p(codes[b][w].data_ptr()), sp)
                       for w in range(W)])
        cp = (ctypes.c_void_p * W)(*[codes[b][w].data_ptr() for w in range(W)])
        lp = (ctypes.c_void_p * W)(*[levels[b][w].data_ptr() for w in range(W)])
        keep.append((cp, lp))
        a_args.append((ctypes.c_void_p(ctypes.addressof(cp)), ctypes.c_void_p(ctypes.addressof(lp)),
                       ctypes.c_uint32(W), ctypes.c_size_t(n), ctypes.byref(dparams),
                       ctypes.c_void_p(outs[b].data_ptr()), sp))
    quantize, average = L.ogq_quantize, L.ogq_dequantize_average

    def step(i: int):
        b = i % n_buf
        rc = 0
        for a in q_args[b]:
            rc |= quantize(*a)
        rc |= average(*a_args[b])
        if rc:
            raise RuntimeError(f"libogq returned an error status in step {i}")

    def ev():
        return torch.cuda.Event(enable_timing=True)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps ------------------------------------------------------------
    e_begin, e_end = ev(), ev()
    graph = None
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for i in range(args.steps):
                step(args.warmup + i)
        torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e_begin.record(stream)
    if graph is not None:
        graph.replay()
    else:
        for i in range(args.steps):
            step(args.warmup + i)
    e_end.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gpu_ms_per_step = e_begin.elapsed_time(e_end) / args.steps

    # ---- per-kernel launch duration ---------------------------------------------------------------
    # An event recorded between two 18 us kernels costs the queue 1-3 us, so each kernel is timed as K
    # back-to-back launches over the rotating buffers between two HIP events on the launch stream
    # (this agrees with the kernel durations rocprofv3 reports for the same command).
    eq0, eq1, ea0, ea1 = ev(), ev(), ev(), ev()
    eq0.record(stream)
    for i in range(args.steps):
        for a in q_args[i % n_buf]:
            quantize(*a)
    eq1.record(stream)
    torch.cuda.synchronize()
    # The decoder's inputs are the packed streams, 1/32 .. 1/8 of the gradient's size: the sets the step loop rotates
    # over stay in the 256 MB last-level cache, as they do inside a step, where the decoder reads what the quantizer
    # has just written.  The decoder is therefore timed twice: over those sets, and over as many further sets of packed
    # streams and level tables as it takes to hold 512 MB (at most 192; filled by untimed quantize launches), which is
    # what it sees when the streams arrive from elsewhere.  The outputs rotate over the step loop's buffers.
    codes_per_set = W * n_words * 8
    n_sets = max(n_buf, min(192, -(-(512 << 20) // codes_per_set) + 1))
    d_args = list(a_args)
    for s in range(n_buf, n_sets):
        lv_s = [torch.empty(n_levels + 4, dtype=torch.float32, device=dev) for _ in range(W)]
        cd_s = [torch.empty(n_words + 2, dtype=torch.int64, device=dev) for _ in range(W)]
        for w in range(W):
            rc = quantize(ctypes.c_void_p(grads[s % n_buf][w].data_ptr()), ctypes.c_size_t(n), ctypes.byref(params[w]),
                          ctypes.c_void_p(lv_s[w].data_ptr()), ctypes.c_void_p(cd_s[w].data_ptr()), sp)
            if rc:
                raise RuntimeError("libogq returned an error status while filling the decoder's inputs")
        cp = (ctypes.c_void_p * W)(*[x.data_ptr() for x in cd_s])
        lp = (ctypes.c_void_p * W)(*[x.data_ptr() for x in lv_s])
        keep.append((cp, lp, lv_s, cd_s))
        d_args.append((ctypes.c_void_p(ctypes.addressof(cp)), ctypes.c_void_p(ctypes.addressof(lp)),
                       ctypes.c_uint32(W), ctypes.c_size_t(n), ctypes.byref(dparams),
                       ctypes.c_void_p(outs[s % n_buf].data_ptr()), sp))
    torch.cuda.synchronize()
    for i in range(min(n_sets, 8)):
        average(*d_args[i])
    ec0, ec1 = ev(), ev()
    ec0.record(stream)
    for i in range(args.steps):
        average(*d_args[i % n_sets])
    ec1.record(stream)
    torch.cuda.synchronize()
    # ... and over the step loop's own sets, i.e. with the packed streams where a step leaves them
    ea0.record(stream)
    for i in range(args.steps):
        average(*a_args[i % n_buf])
    ea1.record(stream)
    torch.cuda.synchronize()
    a_cold = ec0.elapsed_time(ec1) / args.steps  # ms per decode-average launch on cold packed streams
    q_avg = eq0.elapsed_time(eq1) / (args.steps * W)  # ms per quantize launch
    a_avg = ea0.elapsed_time(ea1) / args.steps        # ms per decode-average launch
    q_bytes, a_bytes = algorithmic_bytes(n, d, bits, W, ogq.ogq_levels_per_bucket(params[0]))
    q_gbs = q_bytes / (q_avg * 1e-3) / 1e9
    a_gbs = a_bytes / (a_avg * 1e-3) / 1e9

    # practical ceilings of this device on the same buffers: a pure streaming read, and a plain copy
    # (the copy is also the kernel of known size that calibrates the hardware traffic counters)
    sink = torch.empty(ogq.binding.PROBE_SINK_FLOATS, dtype=torch.float32, device=dev)
    reps = 40

    def timed(fn):
        for i in range(5):
            fn(i)
        a, b = ev(), ev()
        a.record(stream)
        for i in range(reps):
            fn(i)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e-3

    probe_gbs = 4 * n / timed(lambda i: ogq.ogq_probe_read(grads[i % n_buf][0], sink)) / 1e9
    copy_gbs = 8 * (n - n % 4) / timed(lambda i: ogq.ogq_probe_copy(grads[i % n_buf][0], outs[(i + 1) % n_buf])) / 1e9

    two_level_means = wl.scheme in (synth.BINGRAD_B, synth.SCALED_SIGN)
    if not two_level_means and d in (64, 128):
        quant_name = "even_small_kernel" if wl.scheme == synth.EVEN else "sorted_small_kernel"
    elif not two_level_means:
        quant_name = "orq_quantize_kernel" if d <= 2048 else "orq_team_kernel"
    elif d > 2048:
        quant_name = "bingrad_team_kernel"
    elif wl.clip_factor == 0 and 2048 % d == 0 and d < 2048 and (d <= 256 or n // 2048 >= 2048):
        quant_name = "bingrad_chunk_kernel"
    else:
        quant_name = "bingrad_quantize_kernel"
    # The wave-per-bucket ORQ / BinGrad-pb kernel issues ~110 VALU instructions per element (Philox, exact
    # rank selection): it is bound by VALU issue, not by HBM; its line still prices it against the HBM peak.
    dominant_is_quant = q_avg * W >= a_avg
    roof = {
        "bound": "hbm", "kernel": quant_name if dominant_is_quant else "dequantize_average_kernel",
        "achieved": round(q_gbs if dominant_is_quant else a_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round((q_gbs if dominant_is_quant else a_gbs) / HBM_PEAK_GBS, 4),
        "traffic": read_traffic_note(f"{args.workload}:{quant_name if dominant_is_quant else 'dequantize_average_kernel'}"),
        "algorithmic_bytes_per_launch": q_bytes if dominant_is_quant else a_bytes,
        "avg_launch_us": round((q_avg if dominant_is_quant else a_avg) * 1e3, 2),
    }
    cold = {"cold_avg_launch_us": round(a_cold * 1e3, 2), "cold_achieved": round(a_bytes / (a_cold * 1e-3) / 1e9, 1),
            "cold_frac": round(a_bytes / (a_cold * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "cold_input_sets": n_sets}
    other = {
        "kernel": "dequantize_average_kernel" if dominant_is_quant else quant_name,
        "achieved": round(a_gbs if dominant_is_quant else q_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round((a_gbs if dominant_is_quant else q_gbs) / HBM_PEAK_GBS, 4),
        "traffic": read_traffic_note(f"{args.workload}:{'dequantize_average_kernel' if dominant_is_quant else quant_name}"),
        "algorithmic_bytes_per_launch": a_bytes if dominant_is_quant else q_bytes,
        "avg_launch_us": round((a_avg if dominant_is_quant else q_avg) * 1e3, 2),
    }

    (other if dominant_is_quant else roof).update(cold)  # the decoder's entry also carries its cold-stream figures

    # VALU instructions per wavefront of the quantize kernel, from rocprofv3 --pmc SQ_INSTS_VALU / SQ_WAVES
    # (profiles/valu_instructions.txt), priced against 78.6 T lane-operations/s (256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz)
    valu_per_wave = read_note("valu_instructions.txt", f"{args.workload}:{quant_name}")
    alu = None
    if valu_per_wave is not None and not two_level_means:
        waves_per_bucket = 1 if d <= 2048 else 2 if d <= 8192 else 4 if d <= 16384 else 8
        lane_ops = valu_per_wave * 64 * waves_per_bucket * ((n + d - 1) // d)
        achieved = lane_ops / (q_avg * 1e-3) / 1e12
        alu = {"bound": "alu", "kernel": quant_name, "achieved": round(achieved, 2), "peak": 78.6,
               "unit": "T lane-op/s", "frac": round(achieved / 78.6, 4), "valu_instructions_per_wavefront": valu_per_wave}

    result = {
        "metric": "quantize+pack GB/s of fp32 gradient (fraction of HBM peak); dequant-avg GB/s",
        "value": round(grad_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s of fp32 gradient through quantize+pack+decode-average",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "gpu_ms_per_step": round(gpu_ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 data, f64 sums", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.description}", "n": n, "bucket_size": d, "bits": bits,
                   "workers": W, "level_iters": wl.level_iters, "clip_factor": wl.clip_factor,
                   "input_buffers": n_buf, "decoder_input_sets": n_sets,
                   "launch": "one HIP graph of the K steps" if args.graph else "direct"},
        "elements_per_s": round(n * W / (ms_per_step * 1e-3), 1),
        "quantize_gbs_fp32_in": round(4 * n / (q_avg * 1e-3) / 1e9, 1),
        "dequant_avg_gbs_fp32_out": round(4 * n / (a_avg * 1e-3) / 1e9, 1),
        "read_probe_gbs": round(probe_gbs, 1),
        "copy_probe_gbs_read_plus_write": round(copy_gbs, 1),
        "roofline": roof,
        "roofline_other_kernel": other,
    }
    if alu:
        result["alu"] = alu

    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.threads()
        g0 = host  # the workload's own gradient(s)
        # bounded sample: whole gradients for the small workloads, a prefix for the big ones
        sample_n = n if wl.scheme == synth.BINGRAD_B else min(n, 4_194_304)
        sample_n -= sample_n % d
        t_cpu, reps_cpu = 0.0, 0
        while t_cpu < args.cpu_seconds and reps_cpu < 1000:
            c0 = time.perf_counter()
            q = [oracle.quantize(g0[w][:sample_n], d, bits, wl.scheme, wl.level_iters, wl.philox_seed(w), 0,
                                 wl.clip_factor) for w in range(W)]
            oracle.dequantize_average([x[1] for x in q], [x[0] for x in q], sample_n, d, bits,
                                      ogq.ogq_levels_per_bucket(params[0]))
            t_cpu += time.perf_counter() - c0
            reps_cpu += 1
        # the same oracle on one thread, on a shorter prefix of worker 0's gradient
        one_n = min(sample_n, 2_097_152)
        one_n -= one_n % d
        oracle.set_threads(1)
        c0 = time.perf_counter()
        q1 = oracle.quantize(g0[0][:one_n], d, bits, wl.scheme, wl.level_iters, wl.philox_seed(0), 0, wl.clip_factor)
        oracle.dequantize_average([q1[1]], [q1[0]], one_n, d, bits, ogq.ogq_levels_per_bucket(params[0]))
        t_one = time.perf_counter() - c0
        oracle.set_threads(threads)
        result["cpu_baseline"] = {
            "value": round(4 * sample_n * W * reps_cpu / t_cpu / 1e9, 3),
            "unit": "GB/s of fp32 gradient through quantize+pack+decode-average",
            "cores": threads, "kind": "oracle",
            "sample": f"first {sample_n} elements of each worker's gradient of {wl.name}, {reps_cpu} repetitions, "
                      f"{t_cpu:.1f} s, OpenMP over buckets",
            "single_thread_value": round(4 * one_n / t_one / 1e9, 4),
            "single_thread_sample": f"first {one_n} elements of worker 0's gradient, one pass, {t_one:.2f} s",
        }
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
