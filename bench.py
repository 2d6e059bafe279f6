#!/usr/bin/env python3
"""Benchmark of the per-bucket quantization hot path on one MI355X.

A step is one pass of the whole path over one synthetic gradient that is already resident in HBM:
ogq_quantize (statistics, level solve, encode, bit-pack) of every worker's gradient followed by one
ogq_dequantize_average of the packed stream(s).  The default workload is cfg4, the largest single gradient of the
five configurations (ORQ 3-bit on a VGG-19-shaped gradient of 143.7 M fp32, bucket 4096); --workload picks
another one.  Inputs rotate over several distinct buffers (>= 1 GB in total) so that the 256 MB last-level
cache cannot serve repeats.

Prints ONE JSON line.  `value` is the fp32-gradient throughput of the whole step (4*n*workers bytes per step /
time per step); `roofline` prices the dominant kernel's algorithmic bytes per launch against the HBM peak using
HIP-event timings taken on the launch stream (the decoder's entry also carries `cold_*` figures: the same
kernel over packed streams that no cache holds); `per_config` holds the same per-kernel figures for all five
configurations, measured in the same run; `cpu_baseline` is the plain CPU oracle timed on the host cores, with
OpenMP over buckets and on one thread (a reported baseline only).
"""
from __future__ import annotations

import argparse
import ctypes
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published peak
ALU_PEAK_TLANEOPS = 78.6  # 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz (the units of the published 157.3 TFLOP/s fp32 vector figure / 2)
FIVE_CONFIGS = ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5")
WORKLOAD_NAMES = FIVE_CONFIGS + ("pb2", "orq5", "orq3clip", "cfg2clip", "bin512", "sign2", "tern3", "linear5",
                                 "orq3d32k", "orq3d128")


def algorithmic_bytes(n: int, bucket_size: int, bits: int, workers: int, levels_per_bucket: int):
    """Bytes the method must move per launch: quantize reads the gradient once and writes codes and
    levels; decode-average reads every worker's codes and levels and writes the fp32 average."""
    nb = (n + bucket_size - 1) // bucket_size
    codes = ((n + 63) // 64) * bits * 8
    levels = nb * levels_per_bucket * 4
    return 4 * n + codes + levels, workers * (codes + levels) + 4 * n


def read_note(file_name: str, kernel_key: str):
    """A figure recorded from a separate rocprofv3 counter run: `<workload>:<kernel> <value>` lines under
    profiles/ (the counters cannot be read from inside this process)."""
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


def quantize_kernel_name(synth, wl, n: int) -> str:
    d = wl.bucket_size
    two_level_means = wl.scheme in (synth.BINGRAD_B, synth.SCALED_SIGN)
    if not two_level_means and d in (64, 128):
        return "even_small_kernel" if wl.scheme == synth.EVEN else "sorted_small_kernel"
    if not two_level_means:
        return "orq_quantize_kernel" if d <= 2048 else "orq_team_kernel"
    if d > 2048:
        return "bingrad_team_kernel"
    if wl.clip_factor == 0 and 2048 % d == 0 and d < 2048 and (d <= 256 or n // 2048 >= 2048):
        return "bingrad_chunk_kernel"
    return "bingrad_quantize_kernel"


def wavefronts_per_bucket(two_level_means: bool, d: int) -> int:
    if two_level_means:
        return 1
    return 1 if d <= 2048 else 2 if d <= 4096 else 4 if d <= 16384 else 8


class Measurement:
    """Device buffers and marshalled C-ABI arguments of one workload, and the timing loops over them."""

    def __init__(self, name: str, torch, np, ogq, synth, dev, stream, buffers: int = 0, elements: int = 0):
        self.torch, self.ogq = torch, ogq
        self.wl = wl = synth.WORKLOADS[name]
        self.n, self.d, self.bits, self.W = elements or wl.n, wl.bucket_size, wl.bits, wl.workers
        n, d, bits, W = self.n, self.d, self.bits, self.W
        self.grad_bytes = 4 * n * W
        self.n_buf = buffers or max(2, -(-(1 << 30) // self.grad_bytes) + 1)
        if name == "cfg2":
            self.n_buf = max(self.n_buf, 10)
        # Buffer 0 is the workload's own seeded gradient(s); the others hold the same values rolled by a
        # different amount (same distribution, different bytes at every address).
        self.host = [wl.gradient(w, n) for w in range(W)]
        self.grads = [[torch.from_numpy(np.roll(h, 7919 * b) if b else h).to(dev) for h in self.host]
                      for b in range(self.n_buf)]
        self.params = [ogq.make_params(d, bits, wl.scheme, wl.level_iters, wl.philox_seed(w), 0, wl.clip_factor)
                       for w in range(W)]
        self.dparams = ogq.make_params(d, bits, wl.scheme)
        self.n_levels = ogq.ogq_levels_count(n, self.params[0])
        self.n_words = ogq.ogq_codes_bytes(n, self.params[0]) // 8
        self.levels_per_bucket = ogq.ogq_levels_per_bucket(self.params[0])
        self.levels = [[torch.empty(self.n_levels + 4, dtype=torch.float32, device=dev) for _ in range(W)]
                       for _ in range(self.n_buf)]
        self.codes = [[torch.empty(self.n_words + 2, dtype=torch.int64, device=dev) for _ in range(W)]
                      for _ in range(self.n_buf)]
        self.outs = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(self.n_buf)]
        self.dev, self.stream = dev, stream
        # Launch path of the timed loops: the raw C-ABI entry points with every argument marshalled ahead of
        # time, so that the host enqueues faster than the GPU drains and the HIP events that bracket the
        # launches on this stream see back-to-back execution.
        L = ogq.lib()
        self.quantize, self.average = L.ogq_quantize, L.ogq_dequantize_average
        self.sp = sp = ctypes.c_void_p(stream.cuda_stream)
        self.q_args, self.a_args, self.keep = [], [], []
        for b in range(self.n_buf):
            self.q_args.append([(ctypes.c_void_p(self.grads[b][w].data_ptr()), ctypes.c_size_t(n),
                                 ctypes.byref(self.params[w]), ctypes.c_void_p(self.levels[b][w].data_ptr()),
                                 ctypes.c_void_p(self.codes[b][w].data_ptr()), sp) for w in range(W)])
            self.a_args.append(self._average_args(self.codes[b], self.levels[b], self.outs[b]))
        self.q_bytes, self.a_bytes = algorithmic_bytes(n, d, bits, W, self.levels_per_bucket)
        self.quant_name = quantize_kernel_name(synth, wl, n)
        self.two_level_means = wl.scheme in (synth.BINGRAD_B, synth.SCALED_SIGN)

    def _average_args(self, codes, levels, out):
        W = self.W
        cp = (ctypes.c_void_p * W)(*[x.data_ptr() for x in codes])
        lp = (ctypes.c_void_p * W)(*[x.data_ptr() for x in levels])
        self.keep.append((cp, lp, codes, levels))
        return (ctypes.c_void_p(ctypes.addressof(cp)), ctypes.c_void_p(ctypes.addressof(lp)), ctypes.c_uint32(W),
                ctypes.c_size_t(self.n), ctypes.byref(self.dparams), ctypes.c_void_p(out.data_ptr()), self.sp)

    def step(self, i: int):
        b = i % self.n_buf
        rc = 0
        for a in self.q_args[b]:
            rc |= self.quantize(*a)
        rc |= self.average(*self.a_args[b])
        if rc:
            raise RuntimeError(f"libogq returned an error status in step {i}")

    def event(self):
        return self.torch.cuda.Event(enable_timing=True)

    def time_steps(self, steps: int, warmup: int, graph: bool):
        """W untimed steps, then exactly K timed ones; returns (host ms per step, HIP-event ms per step)."""
        torch = self.torch
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        e_begin, e_end = self.event(), self.event()
        g = None
        if graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=self.stream):
                for i in range(steps):
                    self.step(warmup + i)
            torch.cuda.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e_begin.record(self.stream)
        if g is not None:
            g.replay()
        else:
            for i in range(steps):
                self.step(warmup + i)
        e_end.record(self.stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / steps, e_begin.elapsed_time(e_end) / steps

    def time_kernels(self, steps: int):
        """Average launch duration of each kernel, in ms: quantize; decode-average over the step loop's own packed
        streams (still in the last-level cache, as inside a step); decode-average over cold packed streams.

        An event recorded between two short kernels costs the queue 1-3 us, so each kernel is timed as K
        back-to-back launches over the rotating buffers between two HIP events on the launch stream (this agrees
        with the kernel durations rocprofv3 reports for the same command)."""
        torch, n_buf, W = self.torch, self.n_buf, self.W
        for i in range(min(n_buf, 3)):  # untimed: also fills the packed streams when no step loop ran before
            for a in self.q_args[i]:
                self.quantize(*a)
        e0, e1 = self.event(), self.event()
        e0.record(self.stream)
        for i in range(steps):
            for a in self.q_args[i % n_buf]:
                self.quantize(*a)
        e1.record(self.stream)
        torch.cuda.synchronize()
        q_ms = e0.elapsed_time(e1) / (steps * W)
        # The decoder's inputs are the packed streams, 1/32 .. 1/8 of the gradient's size: the sets the step loop
        # rotates over stay in the 256 MB last-level cache.  For the cold figure the decoder runs over as many
        # further sets of packed streams and level tables as it takes to hold 512 MB (at most 192; filled by untimed
        # quantize launches), which is what it sees when the streams arrive from elsewhere.  The outputs rotate over
        # the step loop's buffers.
        codes_per_set = W * self.n_words * 8
        self.n_sets = n_sets = max(n_buf, min(192, -(-(512 << 20) // codes_per_set) + 1))
        d_args = list(self.a_args)
        for s in range(n_buf, n_sets):
            lv_s = [torch.empty(self.n_levels + 4, dtype=torch.float32, device=self.dev) for _ in range(W)]
            cd_s = [torch.empty(self.n_words + 2, dtype=torch.int64, device=self.dev) for _ in range(W)]
            for w in range(W):
                rc = self.quantize(ctypes.c_void_p(self.grads[s % n_buf][w].data_ptr()), ctypes.c_size_t(self.n),
                                   ctypes.byref(self.params[w]), ctypes.c_void_p(lv_s[w].data_ptr()),
                                   ctypes.c_void_p(cd_s[w].data_ptr()), self.sp)
                if rc:
                    raise RuntimeError("libogq returned an error status while filling the decoder's inputs")
            d_args.append(self._average_args(cd_s, lv_s, self.outs[s % n_buf]))
        torch.cuda.synchronize()
        for i in range(min(n_sets, 8)):
            self.average(*d_args[i])
        e0, e1 = self.event(), self.event()
        e0.record(self.stream)
        for i in range(steps):
            self.average(*d_args[i % n_sets])
        e1.record(self.stream)
        torch.cuda.synchronize()
        cold_ms = e0.elapsed_time(e1) / steps
        e0, e1 = self.event(), self.event()
        e0.record(self.stream)
        for i in range(steps):
            self.average(*self.a_args[i % n_buf])
        e1.record(self.stream)
        torch.cuda.synchronize()
        warm_ms = e0.elapsed_time(e1) / steps
        return q_ms, warm_ms, cold_ms

    def kernel_entries(self, q_ms: float, warm_ms: float, cold_ms: float, workload: str):
        """Roofline entries (HBM bound) of the quantize kernel and of the decoder."""
        def entry(kernel, nbytes, ms):
            gbs = nbytes / (ms * 1e-3) / 1e9
            traffic = read_note("hbm_traffic.txt", f"{workload}:{kernel}")
            e = {"bound": "hbm", "kernel": kernel, "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                 "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic,
                 "algorithmic_bytes_per_launch": nbytes, "avg_launch_us": round(ms * 1e3, 2)}
            if traffic is not None:
                e["traffic_source"] = "profiles/hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this workload (recorded, not measured in this run)"
            return e
        quant = entry(self.quant_name, self.q_bytes, q_ms)
        dec = entry("dequantize_average_kernel", self.a_bytes, warm_ms)
        cold_gbs = self.a_bytes / (cold_ms * 1e-3) / 1e9
        dec.update({"cold_avg_launch_us": round(cold_ms * 1e3, 2), "cold_achieved": round(cold_gbs, 1),
                    "cold_frac": round(cold_gbs / HBM_PEAK_GBS, 4), "cold_input_sets": self.n_sets})
        return quant, dec

    def alu_entry(self, q_ms: float, workload: str):
        """The quantize kernel against the vector-ALU peak: VALU instructions per wavefront from a recorded
        rocprofv3 --pmc SQ_INSTS_VALU / SQ_WAVES run x 64 lanes; plus, where recorded, the share of its resident
        time in which a SIMD issues VALU instructions (SQ_ACTIVE_INST_VALU x 4 / SQ_BUSY_CU_CYCLES)."""
        valu_per_wave = read_note("valu_instructions.txt", f"{workload}:{self.quant_name}")
        if valu_per_wave is None or self.two_level_means:
            return None
        buckets = (self.n + self.d - 1) // self.d
        lane_ops = valu_per_wave * 64 * wavefronts_per_bucket(self.two_level_means, self.d) * buckets
        achieved = lane_ops / (q_ms * 1e-3) / 1e12
        simds = 256 * 4
        e = {"bound": "alu", "kernel": self.quant_name, "achieved": round(achieved, 2), "peak": ALU_PEAK_TLANEOPS,
             "unit": "T lane-op/s", "frac": round(achieved / ALU_PEAK_TLANEOPS, 4),
             "valu_instructions_per_wavefront": valu_per_wave,
             # the launch time spread over the VALU instructions a SIMD issues: the kernel's own issue rate
             "ns_per_valu_instruction_and_simd": round(q_ms * 1e6 * simds / (lane_ops / 64), 3),
             "source": "profiles/valu_instructions.txt (recorded counter run); every instruction counted as one issue slot, "
                       "although fp64, 32-bit multiply and conversion instructions take about 1.7 slots"}
        busy = read_note("valu_busy.txt", f"{workload}:{self.quant_name}")
        if busy is not None:
            e["valu_busy_frac"] = busy
            e["valu_busy_source"] = "profiles/valu_busy.txt (recorded counter run)"
        return e

    def release(self):
        for attr in ("grads", "levels", "codes", "outs", "keep", "q_args", "a_args", "host"):
            setattr(self, attr, None)
        gc.collect()
        self.torch.cuda.empty_cache()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4", choices=sorted(WORKLOAD_NAMES))
    ap.add_argument("--buffers", type=int, default=0, help="distinct input buffers (0 = enough for 1 GB)")
    ap.add_argument("--elements", type=int, default=0,
                    help="gradient length per worker instead of the workload's own (its recipe at another size, for size scans)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the per-kernel figures of the other four configurations")
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
    stream = torch.cuda.Stream(dev)  # a real (non-null) stream, default priority
    torch.cuda.set_stream(stream)

    # ---- the headline workload: K whole steps, then each kernel on its own -------------------------------
    m = Measurement(args.workload, torch, np, ogq, synth, dev, stream, args.buffers, args.elements)
    wl, n, d, bits, W = m.wl, m.n, m.d, m.bits, m.W
    ms_per_step, gpu_ms_per_step = m.time_steps(args.steps, args.warmup, args.graph)
    q_ms, warm_ms, cold_ms = m.time_kernels(args.steps)
    quant, dec = m.kernel_entries(q_ms, warm_ms, cold_ms, args.workload)
    dominant_is_quant = q_ms * W >= warm_ms

    # practical ceilings of this device on the same buffers: a pure streaming read, and a plain copy
    # (the copy is also the kernel of known size that calibrates the hardware traffic counters)
    sink = torch.empty(ogq.binding.PROBE_SINK_FLOATS, dtype=torch.float32, device=dev)

    def timed(fn, reps=40):
        for i in range(5):
            fn(i)
        a, b = m.event(), m.event()
        a.record(stream)
        for i in range(reps):
            fn(i)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e-3

    probe_gbs = 4 * n / timed(lambda i: ogq.ogq_probe_read(m.grads[i % m.n_buf][0], sink)) / 1e9
    copy_gbs = 8 * (n - n % 4) / timed(lambda i: ogq.ogq_probe_copy(m.grads[i % m.n_buf][0], m.outs[(i + 1) % m.n_buf])) / 1e9

    result = {
        "metric": "quantize+pack GB/s of fp32 gradient (fraction of HBM peak); dequant-avg GB/s",
        "value": round(m.grad_bytes / (ms_per_step * 1e-3) / 1e9, 2),
        "unit": "GB/s of fp32 gradient through quantize+pack+decode-average",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "gpu_ms_per_step": round(gpu_ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 data, f64 sums", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.description}" + (f" (recipe at {n} elements)" if args.elements else ""), "n": n, "bucket_size": d, "bits": bits,
                   "workers": W, "level_iters": wl.level_iters, "clip_factor": wl.clip_factor,
                   "input_buffers": m.n_buf, "decoder_input_sets": m.n_sets,
                   "launch": "one HIP graph of the K steps" if args.graph else "direct"},
        "elements_per_s": round(n * W / (ms_per_step * 1e-3), 1),
        "quantize_gbs_fp32_in": round(4 * n / (q_ms * 1e-3) / 1e9, 1),
        "dequant_avg_gbs_fp32_out": round(4 * n / (warm_ms * 1e-3) / 1e9, 1),
        "read_probe_gbs": round(probe_gbs, 1),
        "copy_probe_gbs_read_plus_write": round(copy_gbs, 1),
        "roofline": quant if dominant_is_quant else dec,
        "roofline_other_kernel": dec if dominant_is_quant else quant,
    }
    alu = m.alu_entry(q_ms, args.workload)
    if alu:
        result["alu"] = alu

    def summary(name, mm, q, warm, cold, step_ms=None):
        qe, de = mm.kernel_entries(q, warm, cold, name)
        row = {"workload": name, "n": mm.n, "workers": mm.W, "bucket_size": mm.d, "bits": mm.bits,
               "quantize_kernel": qe["kernel"], "quantize_us": qe["avg_launch_us"], "quantize_hbm_frac": qe["frac"],
               "decode_us": de["avg_launch_us"], "decode_hbm_frac": de["frac"],
               "decode_cold_us": de["cold_avg_launch_us"], "decode_cold_hbm_frac": de["cold_frac"]}
        if step_ms is not None:
            row["ms_per_step"] = round(step_ms, 5)
            row["value"] = round(mm.grad_bytes / (step_ms * 1e-3) / 1e9, 2)
        return row

    host, params0 = m.host, m.params[0]
    per_config = {args.workload: summary(args.workload, m, q_ms, warm_ms, cold_ms, ms_per_step)}
    m.host = None
    m.release()
    if not args.no_per_config:
        # the other configurations: the same loops, fewer repetitions (their data generation is the slow part)
        k = max(5, min(args.steps, 20))
        for name in FIVE_CONFIGS:
            if name in per_config:
                continue
            mm = Measurement(name, torch, np, ogq, synth, dev, stream)
            step_ms, _ = mm.time_steps(k, 3, False)
            q, warm, cold = mm.time_kernels(k)
            per_config[name] = summary(name, mm, q, warm, cold, step_ms)
            mm.release()
        result["per_config"] = [per_config[name] for name in sorted(per_config)]

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
                                      ogq.ogq_levels_per_bucket(params0))
            t_cpu += time.perf_counter() - c0
            reps_cpu += 1
        # the same oracle on one thread, on a shorter prefix of worker 0's gradient
        one_n = min(sample_n, 2_097_152)
        one_n -= one_n % d
        oracle.set_threads(1)
        c0 = time.perf_counter()
        q1 = oracle.quantize(g0[0][:one_n], d, bits, wl.scheme, wl.level_iters, wl.philox_seed(0), 0, wl.clip_factor)
        oracle.dequantize_average([q1[1]], [q1[0]], one_n, d, bits, ogq.ogq_levels_per_bucket(params0))
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
