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

Prints ONE JSON line.  `roofline` is for the kernel that takes most of the step: achieved =
algorithmic bytes per launch / average kernel duration, against the 8 TB/s HBM peak.  The
duration comes from HIP events that the launch itself stamps at the kernel's begin and end
(mxc_time_next_launch) on every fourth step of the timed region: a launch carrying events costs
a few microseconds more than a plain one, which would otherwise show up in ms_per_step. 
`cpu_baseline` is the CPU oracle timed on the same workload, for context.
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
EVENT_EVERY = 4                # one step in this many has its two launches timed with HIP events


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=3, help="workload number (1..5)")
    ap.add_argument("--format", default="e2m1", help="element format of the timed step, e.g. e2m1")
    ap.add_argument("--ramp", type=float, default=0.15,
                    help="seconds of untimed load before the warm-up steps (clock conditioning)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the untimed format sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--quality-table", action="store_true",
                    help="add the quality proxy (SQNR of the reduced output) for every element "
                         "format, block size and scale width to the JSON line")
    ap.add_argument("--cpu-rows", type=int, default=0, help="rows per partial for the oracle timing")
    return ap.parse_args()


def parse_format(s):
    s = s.lower()
    return int(s[1]), int(s[3])


def algorithmic_bytes(fmt, tp, tokens, hidden):
    """Bytes the method itself must move, per launch: (quantize, dequant-reduce)."""
    n = tokens * hidden
    packed = n * fmt.bits / 8 + n * 1 / fmt.block          # codes + one scale byte per block
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


def quality_table(mxc, torch, xs, T, H):
    """Quality proxy over the paper's whole parameter list (Method: element type, block size,
    scale type): SQNR in dB of the compressed TP reduction against the uncompressed sum of the
    same synthetic partials.  It stands in for the perplexity tables (Model Evaluation and the
    appendix ablation), which need models and data.  The error is computed with plain torch
    outside the library."""
    exact = xs[0].float()
    for t in xs[1:]:
        exact += t.float()
    power = float(exact.double().pow(2).sum())
    out = torch.empty((T, H), dtype=torch.float32, device="cuda")
    table = {}
    elements = [(1, 1), (1, 2), (2, 1), (1, 3), (2, 2), (3, 1), (1, 4), (2, 3), (3, 2)]
    for (fx, fy) in elements:
        for fb in (8, 16, 32):
            for fs in (8, 7, 6, 5, 4):
                f = mxc.Format(fx, fy, fb, fs)
                codes, scales = mxc.quantize_batched(f, xs)
                mxc.dequant_reduce(f, codes, scales, T, H, out=out)
                err = float((out - exact).double().pow(2).sum())
                table[f"e{fx}m{fy}_b{fb}_s{fs}"] = {
                    "effective_bits": mxc.effective_bits(f),
                    "sqnr_db": 10.0 * float(np.log10(power / err)) if err > 0 else float("inf")}
                del codes, scales
    return table


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
    stream = torch.cuda.current_stream()

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
        if ev: mxc.time_next_launch(ev[0], ev[1])
        q_launch[i % PERIOD]()
        if ev: mxc.time_next_launch(ev[2], ev[3])
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

    # ---- timed region ----------------------------------------------------------------------
    # A launch that carries events costs about 5 us more than a plain one, so only every
    # EVENT_EVERY-th step of the timed region is instrumented; all steps count for ms_per_step.
    timed_steps = range(0, args.steps, EVENT_EVERY)
    events = {i: [torch.cuda.Event(enable_timing=True) for _ in range(4)] for i in timed_steps}
    for ev in events.values():
        for e in ev:
            e.record(stream)                # creates the HIP event; the launch re-stamps it
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events.get(i))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    q_all = [e[0].elapsed_time(e[1]) for e in events.values()]
    r_all = [e[2].elapsed_time(e[3]) for e in events.values()]
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
                "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": ms,
                "median_launch_ms": float(np.median(samples)),
                "min_launch_ms": float(np.min(samples)), "launches_timed": len(samples)}

    rq, rr = roof("quantize_kernel", q_bytes, q_all), roof("dequant_reduce_kernel", r_bytes, r_all)
    dominant = rq if q_ms >= r_ms else rr

    result = {
        # `value` is the whole step (quantize + dequant-reduce); the two kernels' own rates and
        # fractions of the HBM peak are under "kernels"
        "metric": "quantize / dequant-reduce GB/s (bf16 in) and % of HBM peak, 1\u00d7 MI355X",
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

    # ---- untimed extras: copy ceiling and the other element formats of the configuration ----
    if not args.no_sweep:
        def time_calls(fn, n=50, warm=100):
            for i in range(warm):
                fn(i)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for i in range(n):
                fn(i)
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / n
        src = [torch.empty(512 << 20, dtype=torch.uint8, device="cuda") for _ in range(2)]
        dst = [torch.empty(512 << 20, dtype=torch.uint8, device="cuda") for _ in range(2)]
        for s in src:
            s.zero_()
        cms = time_calls(lambda i: mxc.copy_probe(dst[i % 2], src[i % 2]))
        copy_gbs = 2 * (512 << 20) / (cms * 1e-3) / 1e9
        result["copy_ceiling"] = {"GBps": copy_gbs, "frac_of_peak": copy_gbs / HBM_PEAK_GBS,
                                  "bytes_moved": 2 * (512 << 20)}
        for k in result["kernels"].values():
            k["frac_of_copy_ceiling"] = k["achieved"] / copy_gbs
        del src, dst
        sweep = {}
        for (fx, fy, fb, fs) in w.formats:
            f = mxc.Format(fx, fy, fb, fs)
            ps = [packed_set(f) for _ in range(R)]
            for i in range(R):
                mxc.quantize_batched(f, x_sets[0], *ps[i])
            qb, rb = algorithmic_bytes(f, N, T, H)
            ql, dl = make_launches(f, ps)
            qms = time_calls(lambda i: ql[i % PERIOD]())
            rms = time_calls(lambda i: dl[i % PERIOD]())
            # quality proxy on the synthetic tensors (the paper's perplexity tables need models
            # and data): error of the reduced output against the uncompressed sum, plain torch
            dl[0]()
            exact = x_sets[0][0].float()
            for r in range(1, N):
                exact += x_sets[0][r].float()
            err = (outs[0] - exact).double()
            sqnr = 10.0 * float(torch.log10(exact.double().pow(2).sum() / err.pow(2).sum()))
            del exact, err
            sweep[f"e{fx}m{fy}_b{fb}"] = {
                "compression_ratio": 16 / mxc.effective_bits(f),
                "reduced_output_sqnr_db": sqnr,
                "quantize": {"ms": qms, "GBps_bf16": bf16_bytes / qms / 1e6,
                             "hbm_GBps": qb / qms / 1e6, "frac": qb / qms / 1e6 / HBM_PEAK_GBS,
                             "frac_of_copy": qb / qms / 1e6 / copy_gbs},
                "dequant_reduce": {"ms": rms, "GBps_bf16": bf16_bytes / rms / 1e6,
                                   "hbm_GBps": rb / rms / 1e6, "frac": rb / rms / 1e6 / HBM_PEAK_GBS,
                                   "frac_of_copy": rb / rms / 1e6 / copy_gbs},
            }
            del ps
        # requantize (extension): every 1/N row chunk of the reduced tensor, one launch per chunk
        # as the ranks would issue them, and the whole tensor in one launch (tp = 1) to show the
        # kernel's streaming rate without the launch gaps
        f = mxc.Format(*w.formats[-1])
        red = outs[0]
        cb, sb = mxc.packed_sizes(f, T // N, H)
        cc = [torch.empty(cb, dtype=torch.uint8, device="cuda") for _ in range(N)]
        sc = [torch.empty(sb, dtype=torch.uint8, device="cuda") for _ in range(N)]
        rl = [mxc.prepare_requantize_chunk(f, red, N, c, cc[c], sc[c]) for c in range(N)]
        def requant_all(i):
            for l in rl:
                l()
        ms = time_calls(requant_all)
        nb = T * H * 4 + N * (cb + sb)
        sweep["requantize_%d_chunks_%d_launches" % (N, N)] = {
            "ms": ms, "hbm_GBps": nb / ms / 1e6, "frac": nb / ms / 1e6 / HBM_PEAK_GBS}
        cbw, sbw = mxc.packed_sizes(f, T, H)
        reds = outs[:3]
        cw = [torch.empty(cbw, dtype=torch.uint8, device="cuda") for _ in range(3)]
        sw = [torch.empty(sbw, dtype=torch.uint8, device="cuda") for _ in range(3)]
        wl = [mxc.prepare_requantize_chunk(f, reds[k], 1, 0, cw[k], sw[k]) for k in range(3)]
        ms = time_calls(lambda i: wl[i % 3]())
        sweep["requantize_whole_tensor_f32"] = {
            "ms": ms, "hbm_GBps": nb / ms / 1e6, "frac": nb / ms / 1e6 / HBM_PEAK_GBS}
        # fused dequant-reduce + requantize of one rank's chunk (N compressed chunk copies in, one
        # compressed chunk out), and of the whole tensor in one launch to show the streaming rate
        fsets = [packed_set(f) for _ in range(R)]
        for i in range(R):
            mxc.quantize_batched(f, x_sets[0], *fsets[i])
        n_rows = T // N
        fl = [mxc.prepare_dequant_reduce_requantize(
                  f, [c[:n_rows] for c in fsets[k][0]], [s_[:n_rows] for s_ in fsets[k][1]],
                  n_rows, H, cc[0], sc[0]) for k in range(R)]
        ms = time_calls(lambda i: fl[i % R]())
        nbf = N * (cb + sb) + cb + sb
        sweep["fused_reduce_requantize_one_chunk"] = {
            "ms": ms, "hbm_GBps": nbf / ms / 1e6, "frac": nbf / ms / 1e6 / HBM_PEAK_GBS}
        fw = [mxc.prepare_dequant_reduce_requantize(f, fsets[k][0], fsets[k][1], T, H, cw[k], sw[k])
              for k in range(R)]
        ms = time_calls(lambda i: fw[i % R]())
        nbw = N * (cbw + sbw) + cbw + sbw
        sweep["fused_reduce_requantize_whole_tensor"] = {
            "ms": ms, "hbm_GBps": nbw / ms / 1e6, "frac": nbw / ms / 1e6 / HBM_PEAK_GBS}
        # the reduction as the paper's Profiling section words it: the worker's own partial raw,
        # the other N-1 decoded, bf16 out (the dtype the next layer consumes); and the
        # rank-consistent all-decoded form with bf16 out
        # eight bf16 outputs (the two halves of each float32 buffer) keep the rotation at 512 MiB
        outs16 = [o.view(-1).view(torch.bfloat16)[h * T * H:(h + 1) * T * H].view(T, H)
                  for o in outs for h in (0, 1)]
        NOUT16 = len(outs16)
        for (fx, fy, fb, fs) in w.formats:
            f = mxc.Format(fx, fy, fb, fs)
            ps = [packed_set(f) for _ in range(R)]
            for i in range(R):
                mxc.quantize_batched(f, x_sets[0], *ps[i])
            cbk, sbk = mxc.packed_sizes(f, T, H)
            dl16 = [mxc.prepare_dequant_reduce(f, *ps[i % R], T, H, outs16[i % NOUT16])
                    for i in range(2 * PERIOD)]
            ms = time_calls(lambda i: dl16[i % (2 * PERIOD)]())
            nb16 = N * (cbk + sbk) + T * H * 2
            sweep[f"dequant_reduce_bf16_out_e{fx}m{fy}"] = {
                "ms": ms, "hbm_GBps": nb16 / ms / 1e6, "frac": nb16 / ms / 1e6 / HBM_PEAK_GBS}
            ms = time_calls(lambda i: mxc.dequant_reduce_own(
                f, i % N, x_sets[i % 2][i % N], ps[i % R][0], ps[i % R][1], out=outs16[i % NOUT16]))
            nbo = (N - 1) * (cbk + sbk) + T * H * 2 + T * H * 2
            sweep[f"dequant_reduce_own_raw_bf16_out_e{fx}m{fy}"] = {
                "ms": ms, "hbm_GBps": nbo / ms / 1e6, "frac": nbo / ms / 1e6 / HBM_PEAK_GBS}
            del ps, dl16
        # the paper's own profiled input sizes are a few hundred tokens (Table 3: 2x64 ... 16x256):
        # one rank's quantize and the N-way reduce at 256 tokens, where a call is launch-bound
        f = mxc.Format(2, 1, 32, 8)
        Ts = 256
        xs_small = [x_sets[0][r][:Ts] for r in range(N)]
        cbs, sbs = mxc.packed_sizes(f, Ts, H)
        cs_small = [torch.empty((Ts, cbs // Ts), dtype=torch.uint8, device="cuda") for _ in range(N)]
        ss_small = [torch.empty((Ts, sbs // Ts), dtype=torch.uint8, device="cuda") for _ in range(N)]
        out_small = torch.empty((Ts, H), dtype=torch.float32, device="cuda")
        q1 = mxc.prepare_quantize_batched(f, xs_small[:1], cs_small[:1], ss_small[:1])
        qn = mxc.prepare_quantize_batched(f, xs_small, cs_small, ss_small)
        rn = mxc.prepare_dequant_reduce(f, cs_small, ss_small, Ts, H, out_small)
        qn()
        def small_step(i):
            qn()
            rn()
        eager_us = time_calls(small_step) * 1e3
        # the same step recorded once into a HIP graph and replayed (the library never allocates
        # or synchronises, so its calls can be captured)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(10):
                small_step(0)
        graph_us = time_calls(lambda i: graph.replay(), n=20, warm=20) * 1e3 / 10
        sweep["paper_sized_256_tokens_e2m1"] = {
            "quantize_one_partial_us": time_calls(lambda i: q1()) * 1e3,
            "dequant_reduce_%d_partials_us" % N: time_calls(lambda i: rn()) * 1e3,
            "step_quantize_%d_plus_reduce_eager_us" % N: eager_us,
            "step_quantize_%d_plus_reduce_graph_replay_us" % N: graph_us,
        }
        result["sweep"] = sweep

    if args.quality_table:
        result["quality_table"] = quality_table(mxc, torch, x_sets[0], T, H)

    if not args.no_cpu_baseline:
        rows = args.cpu_rows or min(T, 4096)
        result["cpu_baseline"] = cpu_baseline(w, x, y, host_parts, rows)
    else:
        result["cpu_baseline"] = None

    print(json.dumps(result))


if __name__ == "__main__":
    main()
