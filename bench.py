#!/usr/bin/env python3
"""Benchmark of the compression hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input at the
Llama-70B-shaped configuration: the 8 tensor-parallel partials (bf16 [4096 x 8192] each) are
block-quantized in one batched launch, and 8 compressed partials are decoded and summed to
float32 by one launch.  The metric is GB/s of bf16 activations processed per step (the
512 MiB of partials that go through both kernels) with all inputs resident in HBM.

So that no kernel reads data another kernel has just left in the 256 MB last-level cache, the
packed buffers rotate over three sets (a step quantizes into one set and reduces the set that
was written two steps earlier), the bf16 inputs alternate between two copies and the reduced
outputs rotate over four buffers.

Prints ONE JSON line.  `value` and `ms_per_step` are wall-clock over the K timed steps, which
carry no instrumentation.  `roofline` is for the kernel that takes most of the step: achieved =
algorithmic bytes per launch / average kernel duration, against the 8 TB/s HBM peak.  The
durations come from an instrumented pass right after the timed region: the same steps again,
every launch stamping a pair of HIP events at the kernel's own begin and end
(mxc_time_next_launch), at least 50 launches per kernel whatever --steps is.  `cpu_baseline` is
the CPU oracle timed on the same workload, for context.  The untimed `sweep` adds the other
element formats of the configuration, the other forms of the reduction, and the requantize
pipelines of the two larger configurations and configuration 2, each kernel timed the same way.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MIN_TIMED_LAUNCHES = 50        # per kernel, in the instrumented pass and in the sweep
QUANTIZE_KERNEL = "quantize_kernel"


def reduce_kernel(x, y, tp, tokens, hidden):
    """Name of the kernel mxc_dequant_reduce launches (as rocprofv3 prints it): E2M1 tensors of
    whole 1024-element wave tiles, up to 6144 x 8192 elements, with 6 to 8 partials take the
    half-chunk form."""
    n = tokens * hidden
    if (x, y) == (2, 1) and 6 <= tp <= 8 and n % 1024 == 0 and n <= 6144 * 8192:
        return "dequant_reduce_half_kernel"
    return "dequant_reduce_tile_kernel"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=3, help="workload number (1..5)")
    ap.add_argument("--format", default="e2m1", help="element format of the timed step, e.g. e2m1")
    ap.add_argument("--ramp", type=float, default=0.15,
                    help="seconds of untimed load before the warm-up steps (clock conditioning)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the untimed sweep")
    ap.add_argument("--no-pipelines", action="store_true",
                    help="skip the requantize pipelines of configurations 4 and 5 in the sweep")
    ap.add_argument("--format-table", action="store_true",
                    help="also time quantize and dequant-reduce for every element type of the Method list "
                         "(blocks of 32 and 8)")
    ap.add_argument("--one-rank", action="store_true",
                    help="also time what one rank of the group launches per all-reduce: the quantize of a "
                         "single partial and the decode of a single compressed copy")
    ap.add_argument("--tp-sweep", action="store_true",
                    help="add the reduce kernel's rate from 1, 2, 4, ... of the partials to the sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quality-table", action="store_true",
                    help="add the quality proxy (SQNR of the reduced output) for every element "
                         "format, block size and scale width to the JSON line")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows per partial for the oracle timing")
    return ap.parse_args()


def parse_format(s):
    s = s.lower()
    return int(s[1]), int(s[3])


def packed_bytes(fmt, tokens, hidden):
    """Code bytes + scale bytes of one [tokens x hidden] tensor."""
    n = tokens * hidden
    return n * fmt.bits / 8 + n / fmt.block * fmt.scale_bits / 8


def algorithmic_bytes(fmt, tp, tokens, hidden):
    """Bytes the method itself must move, per launch: (quantize, dequant-reduce to float32)."""
    n = tokens * hidden
    packed = packed_bytes(fmt, tokens, hidden)
    return tp * (n * 2 + packed), tp * packed + n * 4


def read_traffic(workload, kernel, fmt_name):
    """HBM traffic per launch measured with rocprofv3 --pmc (committed under profiles/)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    key = f"{workload}.{kernel}.{fmt_name}"
    for line in open(path):
        line = line.strip()
        if line.startswith("#") or "=" not in line:
            continue
        k, v = [t.strip() for t in line.split("=", 1)]
        if k == key:
            return float(v.split()[0])
    return None


def cpu_baseline(w, x, y, host_parts, rows, reps=3):
    """The oracle, as it is, on a bounded sample of the same workload (host cores): `reps`
    passes of quantize + dequant-reduce over the sample, mean time per pass."""
    import oracle
    fo = oracle.Format(x, y, 32, 8)
    oracle.lib()
    parts = [np.ascontiguousarray(p[:rows]) for p in host_parts]
    tq = tr = 0.0
    for _ in range(reps):
        t0 = time.perf_counter()
        cs, ss = [], []
        for p in parts:
            c, s = oracle.quantize_bf16(fo, p)
            cs.append(c)
            ss.append(s)
        t1 = time.perf_counter()
        oracle.dequant_reduce(fo, cs, ss)
        t2 = time.perf_counter()
        tq += (t1 - t0) / reps
        tr += (t2 - t1) / reps
    nbytes = w.tp * rows * w.hidden * 2
    return {
        "value": nbytes / (tq + tr) / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"first {rows} of {w.tokens} rows of each of the {w.tp} partials of the timed "
                  f"workload, quantize + dequant-reduce, e{x}m{y} block 32, mean of {reps} passes",
        "quantize_GBps": nbytes / tq / 1e9, "dequant_reduce_GBps": nbytes / tr / 1e9,
        "seconds": (tq + tr) * reps,
    }


def sqnr_db(torch, out, exact):
    err = (out.double() - exact.double()).pow(2).sum()
    return 10.0 * float(torch.log10(exact.double().pow(2).sum() / err)) if float(err) > 0 else float("inf")


def quality_table(mxc, torch, xs, T, H):
    """Quality proxy over the paper's whole parameter list (Method: element type, block size,
    scale type): SQNR in dB of the compressed TP reduction against the uncompressed sum of the
    same synthetic partials.  It stands in for the perplexity tables (Model Evaluation and the
    appendix ablation), which need models and data.  The error is computed with plain torch
    outside the library."""
    exact = xs[0].float()
    for t in xs[1:]:
        exact += t.float()
    out = torch.empty((T, H), dtype=torch.float32, device="cuda")
    table = {}
    elements = [(1, 1), (1, 2), (2, 1), (1, 3), (2, 2), (3, 1), (1, 4), (2, 3), (3, 2)]
    for (fx, fy) in elements:
        for fb in (8, 16, 32):
            for fs in (8, 7, 6, 5, 4):
                f = mxc.Format(fx, fy, fb, fs)
                codes, scales = mxc.quantize_batched(f, xs)
                mxc.dequant_reduce(f, codes, scales, T, H, out=out)
                table[f"e{fx}m{fy}_b{fb}_s{fs}"] = {
                    "effective_bits": mxc.effective_bits(f), "sqnr_db": sqnr_db(torch, out, exact)}
                del codes, scales
    return table


def format_table(mxc, torch, timer, x_sets, outs, T, H, N):
    """Kernel times of quantize (all N partials) and dequant-reduce (to float32) over the
    element types of the Method list and two block sizes, on the timed workload's tensors; packed
    sets laid out and rotated as in the timed step."""
    table = {}
    for (fx, fy) in [(1, 1), (1, 2), (2, 1), (1, 3), (2, 2), (3, 1), (1, 4), (2, 3), (3, 2)]:
        for fb in (32, 8):
            f = mxc.Format(fx, fy, fb, 8)
            cb, sb = mxc.packed_sizes(f, T, H)
            sets = []
            for _ in range(3):
                buf = torch.empty(N * (cb + sb), dtype=torch.uint8, device="cuda")
                sets.append(([buf[r * (cb + sb): r * (cb + sb) + cb].view(T, cb // T) for r in range(N)],
                             [buf[r * (cb + sb) + cb: (r + 1) * (cb + sb)].view(T, sb // T) for r in range(N)]))
                mxc.quantize_batched(f, x_sets[0], *sets[-1])
            ql = [mxc.prepare_quantize_batched(f, x_sets[k % 2], *sets[k % 3]) for k in range(6)]
            dl = [mxc.prepare_dequant_reduce(f, *sets[k % 3], T, H, outs[k % len(outs)])
                  for k in range(3 * len(outs))]
            table[f"e{fx}m{fy}_b{fb}"] = {
                "effective_bits": mxc.effective_bits(f),
                "quantize": rate(N * (T * H * 2 + cb + sb), timer.each(lambda i: ql[i % len(ql)]())),
                "dequant_reduce": rate(N * (cb + sb) + T * H * 4, timer.each(lambda i: dl[i % len(dl)]())),
            }
            del sets, ql, dl
    return table


class KernelTimer:
    """Durations of single kernels from HIP events that the launches stamp themselves."""

    def __init__(self, mxc, torch):
        self.mxc, self.torch = mxc, torch

    def events(self, n):
        ev = [(self.torch.cuda.Event(enable_timing=True), self.torch.cuda.Event(enable_timing=True))
              for _ in range(n)]
        stream = self.torch.cuda.current_stream()
        for a, b in ev:
            a.record(stream)                # creates the HIP event; the launch re-stamps it
            b.record(stream)
        return ev

    def each(self, launch, n=MIN_TIMED_LAUNCHES, warm=30):
        """launch(i) enqueues exactly one kernel: its duration in ms for i = 0..n-1."""
        for i in range(warm):
            launch(i)
        ev = self.events(n)
        self.torch.cuda.synchronize()
        for i, (a, b) in enumerate(ev):
            self.mxc.time_next_launch(a, b)
            launch(i)
        self.torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in ev]

    def group(self, launches, n=MIN_TIMED_LAUNCHES, warm=10):
        """`launches(i)` returns the list of one-kernel callables of repetition i: the sum of
        their kernel durations in ms per repetition."""
        for i in range(warm):
            for l in launches(i):
                l()
        k = len(launches(0))
        ev = self.events(n * k)
        self.torch.cuda.synchronize()
        for i in range(n):
            for j, l in enumerate(launches(i)):
                self.mxc.time_next_launch(*ev[i * k + j])
                l()
        self.torch.cuda.synchronize()
        return [sum(ev[i * k + j][0].elapsed_time(ev[i * k + j][1]) for j in range(k)) for i in range(n)]


def rate(nbytes, samples_ms):
    ms = float(np.mean(samples_ms))
    gbs = nbytes / ms / 1e6
    return {"ms": ms, "median_ms": float(np.median(samples_ms)), "min_ms": float(np.min(samples_ms)),
            "hbm_GBps": gbs, "frac": gbs / HBM_PEAK_GBS, "launches_timed": len(samples_ms)}


def device_partials(w, torch):
    """The workload's recipe (workloads.py) drawn on the device with torch's generator: the same
    channel profile, body values from a different random stream.  For timing only; the parity
    tests use the numpy draws."""
    import workloads
    chan_scale, _, mult = workloads.channel_profile(w)
    prof = torch.from_numpy(chan_scale * mult).cuda()
    xs = []
    for r in range(w.tp):
        g = torch.Generator(device="cuda")
        g.manual_seed(w.seed * 1000 + r + 1)
        body = torch.randn((w.tokens, w.hidden), generator=g, device="cuda", dtype=torch.float32)
        if w.body == "student_t3":
            chi = torch.zeros_like(body)
            for _ in range(3):
                chi += torch.randn((w.tokens, w.hidden), generator=g, device="cuda").pow_(2)
            body /= (chi / 3.0).sqrt_()
            del chi
        body *= prof[None, :]
        xs.append(body.to(torch.bfloat16))
        del body
    return xs


def pipeline_block(mxc, torch, timer, w, fmt_tuple):
    """Quantize -> dequant-reduce -> requantize at one of the larger configurations, each kernel
    timed by its own events: the unfused path (reduce the whole tensor to float32, requantize each
    1/N row chunk) and the fused path (one launch per chunk: N compressed chunk copies in, one
    compressed chunk out)."""
    T, H, N = w.tokens, w.hidden, w.tp
    f = mxc.Format(*fmt_tuple)
    xs = device_partials(w, torch)
    cb, sb = mxc.packed_sizes(f, T, H)
    R = 2 if N * (cb + sb) > (256 << 20) else 3      # sets whose total exceeds the last-level cache
    sets = []
    for _ in range(R):
        buf = torch.empty(N * (cb + sb), dtype=torch.uint8, device="cuda")
        sets.append(([buf[r * (cb + sb): r * (cb + sb) + cb].view(T, cb // T) for r in range(N)],
                     [buf[r * (cb + sb) + cb: (r + 1) * (cb + sb)].view(T, sb // T) for r in range(N)]))
    outs = [torch.empty((T, H), dtype=torch.float32, device="cuda") for _ in range(2)]
    ql = [mxc.prepare_quantize_batched(f, xs, *sets[k]) for k in range(R)]
    dl = [mxc.prepare_dequant_reduce(f, *sets[k], T, H, outs[k % 2]) for k in range(R)]
    for l in ql:
        l()
    n = T * H
    packed = packed_bytes(f, T, H)
    rows = T // N
    ccb, csb = mxc.packed_sizes(f, rows, H)
    cc = [torch.empty(ccb, dtype=torch.uint8, device="cuda") for _ in range(N)]
    cs = [torch.empty(csb, dtype=torch.uint8, device="cuda") for _ in range(N)]
    rq = [[mxc.prepare_requantize_chunk(f, outs[k], N, c, cc[c], cs[c]) for c in range(N)]
          for k in range(2)]
    fu = [[mxc.prepare_dequant_reduce_requantize(
               f, [t[c * rows:(c + 1) * rows] for t in sets[k][0]],
               [t[c * rows:(c + 1) * rows] for t in sets[k][1]], rows, H, cc[c], cs[c])
           for c in range(N)] for k in range(R)]
    q = rate(N * (n * 2 + packed), timer.each(lambda i: ql[i % R]()))
    d = rate(N * packed + n * 4, timer.each(lambda i: dl[i % R]()))
    r = rate(n * 4 + packed, timer.group(lambda i: rq[i % 2]))
    fz = rate((N + 1) * packed, timer.group(lambda i: fu[i % R]))
    block = {
        "workload": w.name, "element": f"e{f.ebits}m{f.mbits}", "block": f.block,
        "data": "synthetic, drawn on the device (same recipe, torch generator)",
        "quantize": q, "dequant_reduce_f32": d,
        "requantize_%d_chunks" % N: r,
        "fused_reduce_requantize_%d_chunks" % N: fz,
        "pipeline_unfused_ms": q["ms"] + d["ms"] + r["ms"],
        "pipeline_fused_ms": q["ms"] + fz["ms"],
    }
    del xs, sets, outs, ql, dl, rq, fu
    torch.cuda.empty_cache()
    return block


def small_config_block(mxc, torch, timer, w, fmt_tuple):
    """Quantize and dequant-reduce of a configuration whose tensors fit the 256 MB last-level
    cache several times over (configuration 2: 4 partials of bf16 [2048 x 4096]): inputs, packed
    sets and outputs each rotate over enough copies (more than 256 MB per kind) that every launch
    still streams from and to HBM."""
    T, H, N = w.tokens, w.hidden, w.tp
    f = mxc.Format(*fmt_tuple)
    n = T * H
    xs0 = device_partials(w, torch)
    RX = (256 << 20) // (N * n * 2) + 2
    RO = (256 << 20) // (n * 4) + 2
    x_sets = [xs0] + [[t.clone() for t in xs0] for _ in range(RX - 1)]
    cb, sb = mxc.packed_sizes(f, T, H)
    RP = (256 << 20) // (N * (cb + sb)) + 2
    sets = []
    for _ in range(RP):
        buf = torch.empty(N * (cb + sb), dtype=torch.uint8, device="cuda")
        sets.append(([buf[r * (cb + sb): r * (cb + sb) + cb].view(T, cb // T) for r in range(N)],
                     [buf[r * (cb + sb) + cb: (r + 1) * (cb + sb)].view(T, sb // T) for r in range(N)]))
    outs = [torch.empty((T, H), dtype=torch.float32, device="cuda") for _ in range(RO)]
    for k in range(RP):
        mxc.quantize_batched(f, xs0, *sets[k])
    ql = [mxc.prepare_quantize_batched(f, x_sets[i % RX], *sets[i % RP]) for i in range(RX * RP)]
    dl = [mxc.prepare_dequant_reduce(f, *sets[i % RP], T, H, outs[i % RO]) for i in range(RP * RO)]
    packed = packed_bytes(f, T, H)
    block = {
        "workload": w.name, "element": f"e{f.ebits}m{f.mbits}", "block": f.block, "tp": N,
        "data": "synthetic, drawn on the device (same recipe, torch generator)",
        "rotation": {"input_sets": RX, "packed_sets": RP, "outputs": RO},
        "quantize": {"kernel": QUANTIZE_KERNEL, **rate(N * (n * 2 + packed), timer.each(lambda i: ql[i % len(ql)]()))},
        "dequant_reduce_f32": {"kernel": reduce_kernel(f.ebits, f.mbits, N, T, H),
                               **rate(N * packed + n * 4, timer.each(lambda i: dl[i % len(dl)]()))},
    }
    del xs0, x_sets, sets, outs, ql, dl
    torch.cuda.empty_cache()
    return block


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no second GPU); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2411_09510_amd as mxc
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    mxc.lib()
    torch.cuda.set_device(0)
    w = workloads.CONFIGS[args.config]
    x, y = parse_format(args.format)
    fmt = mxc.Format(x, y, 32, 8)
    T, H, N = w.tokens, w.hidden, w.tp
    timer = KernelTimer(mxc, torch)

    # ---- inputs, resident in HBM -----------------------------------------------------------
    host_parts = workloads.all_partials_bf16(w)
    def upload():
        return [torch.from_numpy(p.view(np.int16)).view(torch.bfloat16).cuda() for p in host_parts]
    x_sets = [upload(), upload()]
    R = 3
    def packed_set(f):
        """One exchange buffer laid out as an all-gather would leave it: rank r's codes followed
        by its scales, the N ranks back to back."""
        cb, sb = mxc.packed_sizes(f, T, H)
        buf = torch.empty(N * (cb + sb), dtype=torch.uint8, device="cuda")
        codes = [buf[r * (cb + sb): r * (cb + sb) + cb].view(T, cb // T) for r in range(N)]
        scales = [buf[r * (cb + sb) + cb: (r + 1) * (cb + sb)].view(T, sb // T) for r in range(N)]
        return codes, scales
    sets = [packed_set(fmt) for _ in range(R)]
    # four output buffers: with two, the 2 x 128 MiB they occupy would stay resident in the 256 MB
    # last-level cache and the reduce kernel's stores would never reach HBM
    NOUT = 4
    outs = [torch.empty((T, H), dtype=torch.float32, device="cuda") for _ in range(NOUT)]

    # launches with their arguments already marshalled, one per buffer combination
    PERIOD = 12                              # lcm of the rotation lengths 2, 3 and 4
    def make_launches(f, psets):
        q = [mxc.prepare_quantize_batched(f, x_sets[i % 2], *psets[i % R]) for i in range(PERIOD)]
        d = [mxc.prepare_dequant_reduce(f, *psets[(i + 1) % R], T, H, outs[i % NOUT])
             for i in range(PERIOD)]
        return q, d
    q_launch, d_launch = make_launches(fmt, sets)

    def step(i, ev=None):
        # the events are stamped by the two dispatches themselves (begin and end of each kernel),
        # so timing them puts nothing extra on the stream
        if ev: mxc.time_next_launch(ev[0][0], ev[0][1])
        q_launch[i % PERIOD]()
        if ev: mxc.time_next_launch(ev[1][0], ev[1][1])
        d_launch[i % PERIOD]()

    for i in range(R):                      # fill every packed set before anything is reduced
        mxc.quantize_batched(fmt, x_sets[0], *sets[i])
    # Untimed conditioning, independent of --warmup: the GPU's memory and fabric clocks take tens
    # of milliseconds of load to ramp up after the idle set-up phase.
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < args.ramp:
        for i in range(PERIOD):
            step(i)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # ---- timed region: K plain steps -------------------------------------------------------
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # ---- instrumented pass: the same steps, every launch carrying its pair of events -------
    n_inst = max(MIN_TIMED_LAUNCHES, min(args.steps, 96))
    events = [(timer.events(1)[0], timer.events(1)[0]) for _ in range(n_inst)]
    torch.cuda.synchronize()
    for i in range(n_inst):
        step(args.steps + i, events[i])
    torch.cuda.synchronize()
    q_all = [e[0][0].elapsed_time(e[0][1]) for e in events]
    r_all = [e[1][0].elapsed_time(e[1][1]) for e in events]
    q_ms, r_ms = float(np.mean(q_all)), float(np.mean(r_all))

    bf16_bytes = N * T * H * 2
    q_bytes, r_bytes = algorithmic_bytes(fmt, N, T, H)
    value = bf16_bytes / (ms_per_step * 1e-3) / 1e9
    fname = f"e{x}m{y}"

    def roof(kernel, nbytes, samples):
        ms = float(np.mean(samples))
        ach = nbytes / (ms * 1e-3) / 1e9
        return {"kernel": kernel, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                "traffic": read_traffic(w.name, kernel, fname),
                "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/hbm_traffic.txt",
                "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": ms,
                "median_launch_ms": float(np.median(samples)),
                "min_launch_ms": float(np.min(samples)), "launches_timed": len(samples)}

    rq, rr = roof(QUANTIZE_KERNEL, q_bytes, q_all), roof(reduce_kernel(x, y, N, T, H), r_bytes, r_all)
    dominant = rq if q_ms >= r_ms else rr

    result = {
        # `value` is the whole step (quantize + dequant-reduce); the two kernels' own rates and
        # fractions of the HBM peak are under "kernels"
        "metric": "quantize / dequant-reduce GB/s (bf16 in) and % of HBM peak, 1× MI355X",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16 in, u8 codes, f32 accumulate", "data": "synthetic",
        "config": {"workload": w.name, "tp": N, "tokens": T, "hidden": H, "element": fname,
                   "block": 32, "scale": "e8m0",
                   "compression_ratio": 16 / mxc.effective_bits(fmt)},
        "roofline": dominant,
        "kernels": {
            "quantize": {"GBps_bf16": bf16_bytes / (q_ms * 1e-3) / 1e9, **rq},
            "dequant_reduce": {"GBps_bf16": bf16_bytes / (r_ms * 1e-3) / 1e9, **rr},
        },
    }

    # ---- untimed extras --------------------------------------------------------------------
    if not args.no_sweep:
        src = [torch.empty(512 << 20, dtype=torch.uint8, device="cuda") for _ in range(2)]
        dst = [torch.empty(512 << 20, dtype=torch.uint8, device="cuda") for _ in range(2)]
        for s in src:
            s.zero_()
        c = rate(2 * (512 << 20), timer.each(lambda i: mxc.copy_probe(dst[i % 2], src[i % 2])))
        copy_gbs = c["hbm_GBps"]
        result["copy_ceiling"] = {"kernel": "copy_kernel", "GBps": copy_gbs, "frac_of_peak": c["frac"],
                                  "bytes_moved": 2 * (512 << 20), "launches_timed": c["launches_timed"]}
        for k in result["kernels"].values():
            k["frac_of_copy_ceiling"] = k["achieved"] / copy_gbs
        del src, dst
        sweep = {}
        # the element formats of the configuration: both kernels, the quality proxy, and the
        # other forms of the reduction (bf16 out; the paper's own-partial-raw form with bf16 out)
        exact = x_sets[0][0].float()
        for r in range(1, N):
            exact += x_sets[0][r].float()
        # eight bf16 outputs (the two halves of each float32 buffer) keep the rotation at 512 MiB
        outs16 = [o.view(-1).view(torch.bfloat16)[h * T * H:(h + 1) * T * H].view(T, H)
                  for o in outs for h in (0, 1)]
        NOUT16 = len(outs16)
        for (fx, fy, fb, fs) in w.formats:
            f = mxc.Format(fx, fy, fb, fs)
            ps = [packed_set(f) for _ in range(R)]
            for i in range(R):
                mxc.quantize_batched(f, x_sets[0], *ps[i])
            qb, rb = algorithmic_bytes(f, N, T, H)
            pk = packed_bytes(f, T, H)
            ql, dl = make_launches(f, ps)
            entry = {"compression_ratio": 16 / mxc.effective_bits(f)}
            entry["quantize"] = {"kernel": QUANTIZE_KERNEL, **rate(qb, timer.each(lambda i: ql[i % PERIOD]()))}
            entry["dequant_reduce"] = {"kernel": reduce_kernel(fx, fy, N, T, H), **rate(rb, timer.each(lambda i: dl[i % PERIOD]()))}
            for k in ("quantize", "dequant_reduce"):
                entry[k]["GBps_bf16"] = bf16_bytes / entry[k]["ms"] / 1e6
                entry[k]["frac_of_copy"] = entry[k]["hbm_GBps"] / copy_gbs
            # quality proxy on the synthetic tensors (the paper's perplexity tables need models
            # and data): error of the reduced output against the uncompressed sum, plain torch
            dl[0]()
            entry["reduced_output_sqnr_db"] = sqnr_db(torch, outs[0], exact)
            dl16 = [mxc.prepare_dequant_reduce(f, *ps[i % R], T, H, outs16[i % NOUT16])
                    for i in range(2 * PERIOD)]
            entry["dequant_reduce_bf16_out"] = rate(
                N * pk + T * H * 2, timer.each(lambda i: dl16[i % (2 * PERIOD)]()))
            entry["dequant_reduce_own_raw_bf16_out"] = rate(
                (N - 1) * pk + T * H * 2 + T * H * 2,
                timer.each(lambda i: mxc.dequant_reduce_own(
                    f, i % N, x_sets[i % 2][i % N], ps[i % R][0], ps[i % R][1],
                    out=outs16[i % NOUT16])))
            if args.one_rank:
                # what one rank of the group runs per all-reduce: quantize its own partial (one
                # [T x H] tensor; the 2 x N inputs rotate, 1 GiB), and, in the reduce-scatter
                # variant, decode the all-gathered chunks (one compressed copy of the whole tensor)
                q1 = [mxc.prepare_quantize_batched(f, [x_sets[i % 2][(i // 2) % N]], [ps[i % R][0][(i // 2) % N]],
                                                   [ps[i % R][1][(i // 2) % N]]) for i in range(2 * N * R)]
                entry["quantize_one_partial"] = rate(T * H * 2 + pk, timer.each(lambda i: q1[i % len(q1)]()))
                d1 = [mxc.prepare_dequant_reduce(f, [ps[i % R][0][(i // R) % N]], [ps[i % R][1][(i // R) % N]],
                                                 T, H, outs[i % NOUT]) for i in range(N * R * NOUT)]
                entry["decode_one_copy_f32"] = rate(pk + T * H * 4, timer.each(lambda i: d1[i % len(d1)]()))
                d16 = [mxc.prepare_dequant_reduce(f, [ps[i % R][0][(i // R) % N]], [ps[i % R][1][(i // R) % N]],
                                                  T, H, outs16[i % NOUT16]) for i in range(N * R * NOUT16)]
                entry["decode_one_copy_bf16"] = rate(pk + T * H * 2, timer.each(lambda i: d16[i % len(d16)]()))
                del q1, d1, d16
            # requantize (extension): every 1/N row chunk of the reduced tensor, one launch per
            # chunk as the ranks would issue them, and the whole tensor in one launch
            rows = T // N
            ccb, csb = mxc.packed_sizes(f, rows, H)
            cc = [torch.empty(ccb, dtype=torch.uint8, device="cuda") for _ in range(N)]
            sc = [torch.empty(csb, dtype=torch.uint8, device="cuda") for _ in range(N)]
            rl = [[mxc.prepare_requantize_chunk(f, outs[k], N, c_, cc[c_], sc[c_]) for c_ in range(N)]
                  for k in range(NOUT)]
            entry["requantize_%d_chunks" % N] = rate(T * H * 4 + pk, timer.group(lambda i: rl[i % NOUT]))
            cbw, sbw = mxc.packed_sizes(f, T, H)
            cw = [torch.empty(cbw, dtype=torch.uint8, device="cuda") for _ in range(3)]
            sw = [torch.empty(sbw, dtype=torch.uint8, device="cuda") for _ in range(3)]
            wl = [mxc.prepare_requantize_chunk(f, outs[k], 1, 0, cw[k % 3], sw[k % 3]) for k in range(NOUT)]
            entry["requantize_whole_tensor_f32"] = rate(T * H * 4 + pk, timer.each(lambda i: wl[i % NOUT]()))
            # fused dequant-reduce + requantize: the N chunks one launch each, and the whole
            # tensor in one launch to show the streaming rate
            fl = [[mxc.prepare_dequant_reduce_requantize(
                       f, [t[c_ * rows:(c_ + 1) * rows] for t in ps[k][0]],
                       [t[c_ * rows:(c_ + 1) * rows] for t in ps[k][1]], rows, H, cc[c_], sc[c_])
                   for c_ in range(N)] for k in range(R)]
            entry["fused_reduce_requantize_%d_chunks" % N] = rate((N + 1) * pk, timer.group(lambda i: fl[i % R]))
            fw = [mxc.prepare_dequant_reduce_requantize(f, ps[k][0], ps[k][1], T, H, cw[k], sw[k])
                  for k in range(R)]
            entry["fused_reduce_requantize_whole_tensor"] = rate((N + 1) * pk, timer.each(lambda i: fw[i % R]()))
            sweep[f"e{fx}m{fy}_b{fb}"] = entry
            del ps, ql, dl, dl16, rl, wl, fl, fw, cc, sc, cw, sw
        del exact
        # the scale format the paper recommends (Model Evaluation / appendix ablation: E5M0; Table 1
        # is computed with it): same kernels, scales travelling as a 5-bit stream
        for (fx, fy, fb) in ((2, 1, 32), (2, 1, 8)):
            f = mxc.Format(fx, fy, fb, 5)
            cb5, sb5 = mxc.packed_sizes(f, T, H)
            ps = []
            for _ in range(R):
                buf = torch.empty(N * (cb5 + sb5 + 16), dtype=torch.uint8, device="cuda")
                st = cb5 + sb5 + (-(cb5 + sb5)) % 16
                ps.append(([buf[r * st: r * st + cb5].view(T, cb5 // T) for r in range(N)],
                           [buf[r * st + cb5: r * st + cb5 + sb5] for r in range(N)]))
            for i in range(R):
                mxc.quantize_batched(f, x_sets[0], *ps[i])
            pk = packed_bytes(f, T, H)
            ql = [mxc.prepare_quantize_batched(f, x_sets[i % 2], *ps[i % R]) for i in range(PERIOD)]
            dl = [mxc.prepare_dequant_reduce(f, *ps[(i + 1) % R], T, H, outs[i % NOUT]) for i in range(PERIOD)]
            sweep[f"e{fx}m{fy}_b{fb}_e5m0_scale"] = {
                "effective_bits": mxc.effective_bits(f), "compression_ratio": 16 / mxc.effective_bits(f),
                "quantize": {"kernel": QUANTIZE_KERNEL, **rate(N * (T * H * 2 + pk), timer.each(lambda i: ql[i % PERIOD]()))},
                "dequant_reduce": {"kernel": reduce_kernel(fx, fy, N, T, H), **rate(N * pk + T * H * 4, timer.each(lambda i: dl[i % PERIOD]()))},
            }
            del ps, ql, dl
        # how the reduce kernel's rate depends on the number of input streams: the same output
        # (float32 [T x H]) from 1, 2, 4 and all N partials
        if args.tp_sweep:
            f = mxc.Format(*w.formats[0])
            ps = [packed_set(f) for _ in range(R)]
            for i in range(R):
                mxc.quantize_batched(f, x_sets[0], *ps[i])
            pk = packed_bytes(f, T, H)
            by_tp = {}
            for tpn in sorted({1, 2, max(N // 2, 1), N}):
                dl = [mxc.prepare_dequant_reduce(f, ps[i % R][0][:tpn], ps[i % R][1][:tpn], T, H, outs[i % NOUT])
                      for i in range(PERIOD)]
                by_tp["tp%d" % tpn] = rate(tpn * pk + T * H * 4, timer.each(lambda i: dl[i % PERIOD]()))
                del dl
            sweep["dequant_reduce_by_number_of_partials_e%dm%d" % (f.ebits, f.mbits)] = by_tp
            del ps
        # what a launch costs whatever it does: the plain copy kernel on 1 MiB
        small_src = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
        small_dst = torch.zeros(4 << 20, dtype=torch.uint8, device="cuda")
        sweep["launch_floor_copy_1MiB_kernel_us"] = float(np.mean(timer.each(
            lambda i: mxc.copy_probe(small_dst[(i % 4) << 20:((i % 4) + 1) << 20],
                                     small_src[(i % 4) << 20:((i % 4) + 1) << 20])))) * 1e3
        # the paper's own profiled input sizes are a few hundred tokens (Table 3: 2x64 ... 16x256):
        # one rank's quantize and the N-way reduce at 256 tokens, where a call is launch-bound
        f = mxc.Format(2, 1, 32, 8)
        Ts = min(256, T)
        xs_small = [x_sets[0][r][:Ts] for r in range(N)]
        cbs, sbs = mxc.packed_sizes(f, Ts, H)
        cs_small = [torch.empty((Ts, cbs // Ts), dtype=torch.uint8, device="cuda") for _ in range(N)]
        ss_small = [torch.empty((Ts, sbs // Ts), dtype=torch.uint8, device="cuda") for _ in range(N)]
        out_small = torch.empty((Ts, H), dtype=torch.float32, device="cuda")
        q1 = mxc.prepare_quantize_batched(f, xs_small[:1], cs_small[:1], ss_small[:1])
        qn = mxc.prepare_quantize_batched(f, xs_small, cs_small, ss_small)
        rn = mxc.prepare_dequant_reduce(f, cs_small, ss_small, Ts, H, out_small)
        qn()
        stream = torch.cuda.current_stream()
        def wall_us(fn, n=50, warm=100):
            for i in range(warm):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for i in range(n):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n * 1e3
        def small_step():
            qn()
            rn()
        eager_us = wall_us(small_step)
        # the same step recorded once into a HIP graph and replayed (the library never allocates
        # or synchronises, so its calls can be captured)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(10):
                small_step()
        graph_us = wall_us(graph.replay, n=20, warm=20) / 10
        sweep["paper_sized_%d_tokens_e2m1" % Ts] = {
            "quantize_one_partial_kernel_us": float(np.mean(timer.each(lambda i: q1()))) * 1e3,
            "dequant_reduce_%d_partials_kernel_us" % N: float(np.mean(timer.each(lambda i: rn()))) * 1e3,
            "quantize_one_partial_call_us": wall_us(q1),
            "dequant_reduce_%d_partials_call_us" % N: wall_us(rn),
            "step_quantize_%d_plus_reduce_eager_us" % N: eager_us,
            "step_quantize_%d_plus_reduce_graph_replay_us" % N: graph_us,
        }
        result["sweep"] = sweep

    if args.quality_table:
        result["quality_table"] = quality_table(mxc, torch, x_sets[0], T, H)
    if args.format_table:
        result["format_table"] = format_table(mxc, torch, timer, x_sets, outs, T, H, N)

    # ---- the requantize pipelines of the two larger configurations (default workload only) --
    if not args.no_sweep and not args.no_pipelines and args.config == 3:
        del x_sets, sets, outs, q_launch, d_launch
        torch.cuda.empty_cache()
        result["config2"] = small_config_block(mxc, torch, timer, workloads.CONFIGS[2], workloads.CONFIGS[2].formats[0])
        result["pipelines"] = {
            "config4_b16": pipeline_block(mxc, torch, timer, workloads.CONFIGS[4], workloads.CONFIGS[4].formats[0]),
            "config4_b32": pipeline_block(mxc, torch, timer, workloads.CONFIGS[4], workloads.CONFIGS[4].formats[1]),
            "config5": pipeline_block(mxc, torch, timer, workloads.CONFIGS[5], workloads.CONFIGS[5].formats[0]),
        }

    if not args.no_cpu_baseline:
        rows = args.cpu_rows or min(T, 4096)
        result["cpu_baseline"] = cpu_baseline(w, x, y, host_parts, rows)
    else:
        result["cpu_baseline"] = None

    print(json.dumps(result))


if __name__ == "__main__":
    main()
