#!/usr/bin/env python3
"""Benchmark of the butterfly + quantisation hot path on one MI355X.

A step is one pass of the metric's kernel -- the fused forward transform + INT2 quantisation (group 128, fp16
scales) -- over the calibration/prefill batch (n = 4096, 262144 rows of fp16 activations, resident in HBM).
`value` is rows per second through that step; `roofline` describes the same kernel against the roof that binds
it (vector issue; the HBM figures are carried beside it, because the metric asks for them).  Further keys:
`peaks` (what this GPU delivers on a plain copy and on a float32 FMA loop, measured in this run),
`calibration_step` (plan build + fused quantiser + forward + inverse + backward on the same batch, every call
timed), `decode` (latency of the small-batch calls) and the other workloads' figures.

Prints one JSON line.  Everything runs on one GPU; --gpus above 1 is refused.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
VALU_PEAK_TFLOPS = 157.3       # published fp32 vector peak (counts packed fp32 FMAs: two per lane and cycle)
# What this build can issue: 256 compute units x 64 lanes x 2.4 GHz x 2 flops, one unpacked fp32 FMA per lane
# and cycle (packed fp32 instructions are compiled out)
VALU_PEAK_UNPACKED_TFLOPS = 256 * 64 * 2.4e9 * 2 / 1e12
SIMDS = 256 * 4


def alg_bytes_per_row(op: str, n: int, heads: int, itemsize: int, bits: int = 0, group: int = 0,
                      scale_bytes: int = 0) -> int:
    """Bytes the method itself must move per row (twiddles excluded: read once per workgroup)."""
    w = n * heads
    if op in ("fwd", "inv"):
        return 2 * w * itemsize
    if op == "fwd_quant":
        return w * itemsize + w * bits // 8 + (w // group) * scale_bytes
    if op == "bwd":
        return 3 * w * itemsize
    raise ValueError(op)


def alg_flops_per_row(op: str, n: int, heads: int) -> int:
    """3 n log2 n per transform application (paper, table of per-application arithmetic); the
    backward pass runs three cascades plus 4 flops per pair for dtheta."""
    k = n.bit_length() - 1
    one = 3 * n * k * heads
    if op == "bwd":
        return 3 * one + 4 * (n // 2) * k * heads
    return one


def time_kernel(fn, iters: int, warmup: int = 2):
    """Average duration in ms of `fn` (launches on torch's current stream) measured with events on
    that stream.  The clock needs some tens of milliseconds of work to settle (the first dozens of launches of a
    sub-millisecond kernel run up to 1.5x slower), hence the generous warm-up counts of the callers."""
    import torch

    for _ in range(warmup):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return sum(ts) / len(ts), ts[len(ts) // 2], ts[-1]


def cpu_baseline(sample_rows: int):
    """The oracle, as it is, on the host cores: the same step (forward + INT2 quantisation, forward,
    inverse, backward) on a bounded sample of the workload."""
    import numpy as np

    import oracle
    from paper_2509_09679_amd import synth

    chunk = 8192
    t_total = 0.0
    done = 0
    k = 0
    cache = {}
    while done < sample_rows:
        rows = min(chunk, sample_rows - done)
        salt = k % 4  # four distinct seeded chunks, reused in turn (generation is not timed)
        k += 1
        if (salt, rows) not in cache:
            w = synth.make_workload(3, rows=rows, salt=salt)
            cache[(salt, rows)] = (w, np.random.default_rng(salt).standard_normal((rows, w.n)), synth.to_f64(w.x, w.dtype))
        w, dy, x64 = cache[(salt, rows)]
        t0 = time.perf_counter()
        y = oracle.forward(x64, w.theta, w.n)
        codes, scales = oracle.quantize(y.astype(np.float32), w.group, w.bits, w.scale_dtype)
        oracle.pack_codes(codes, w.bits)
        oracle.forward(x64, w.theta, w.n)
        oracle.inverse(y, w.theta, w.n)
        oracle.backward(x64, dy, w.theta, w.n, want_abs=False)
        t_total += time.perf_counter() - t0
        done += rows
    return {"value": done / t_total, "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{done} rows of the n=4096 fp16 workload, same step (fwd+INT2 quant, fwd, inv, bwd), "
                      f"{t_total:.1f} s of wall time on these threads"}


def percentile(ts, q):
    ts = sorted(ts)
    return ts[min(len(ts) - 1, int(q * len(ts)))]


def measured_copy(B, torch, x, y):
    """What the memory system delivers, measured here: a plain copy of the 2 GiB input and a plain read of it (library
    kernels, 16 bytes per lane)."""
    nbytes = x.numel() * x.element_size()
    avg, med, _ = time_kernel(lambda: B.bq_probe_copy(x, y, nbytes), 20, 10)
    sink = torch.empty(B.bq_probe_read_sink_bytes(), dtype=torch.uint8, device=x.device)
    _, med_r, _ = time_kernel(lambda: B.bq_probe_read(x, nbytes, sink), 20, 10)
    return {"measured_copy_GBps": round(2 * nbytes / (med * 1e-3) / 1e9, 1), "copy_bytes": nbytes, "copy_ms": round(med, 4),
            "measured_read_GBps": round(nbytes / (med_r * 1e-3) / 1e9, 1), "read_ms": round(med_r, 4)}


def measured_fma(B, torch, dev):
    """What the vector units deliver, measured here: a float32 FMA loop of independent chains (unpacked instructions,
    as in every kernel of this library)."""
    out = torch.empty(B.bq_probe_fma_out_floats(), dtype=torch.float32, device=dev)
    iters = 4096
    n_fma = B.bq_probe_fma(out, iters)
    avg_f, med_f, _ = time_kernel(lambda: B.bq_probe_fma(out, iters), 10, 3)
    rate = n_fma / (med_f * 1e-3)
    return {"measured_fma_Tlane_ops": round(rate / 1e12, 2), "fma_TFLOPps": round(2 * rate / 1e12, 1),
            "fma_lane_ops_per_launch": n_fma, "fma_ms": round(med_f, 4),
            # lane-FMAs per second / (SIMDs x 16 lanes per cycle) = the clock at which a SIMD would issue one wave
            # instruction every four cycles
            "fma_implied_clock_GHz": round(rate / (SIMDS * 16) / 1e9, 3)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--rows", type=int, default=262144, help="rows of the batch (default: the full workload)")
    ap.add_argument("--cpu-rows", type=int, default=786432, help="rows of the oracle's timed sample (0 = skip)")
    ap.add_argument("--no-extra", action="store_true", help="skip the figures of the other workloads")
    ap.add_argument("--copy-ref", action="store_true",
                    help="also launch one plain device copy of the 2 GiB input (reference for rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE scaling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (rows are independent, so more "
              "GPUs would each take a slice of the rows and add their dtheta once per call)", file=sys.stderr)
        return 2

    import torch

    from paper_2509_09679_amd import binding as B
    from paper_2509_09679_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.lib()  # fails loudly if the HIP library is not built
    dev = "cuda:0"
    torch.cuda.set_device(0)

    cfg = 3
    T = args.rows
    x, theta_h, dy = synth.device_rows(cfg, T, dev, want_dy=True)
    wl = synth.make_workload(cfg, rows=1)
    n, heads, bits, group = wl.n, wl.heads, wl.bits, wl.group
    theta = torch.from_numpy(theta_h).to(dev)
    plan = torch.empty(B.bq_plan_bytes(n, heads), dtype=torch.uint8, device=dev)
    y = torch.empty_like(x)
    codes, scales = B.alloc_quant_outputs(T, n, heads, bits, group, wl.scale_dtype, dev)
    rows = B.make_rows(x, n, heads)
    quant = B.make_quant(bits, group, wl.scale_dtype)
    B.bq_plan_build(theta, n, heads, plan)

    # The plain-copy leg comes first (it also takes the device out of idle before the timed region); the FMA loop,
    # which draws the most power of anything here, runs after the timed region.
    peaks = measured_copy(B, torch, x, y)

    # The other workloads' figures and the five-call calibration step are measured BEFORE the timed region: a
    # calibration run keeps the device busy for minutes, and after a few seconds of work it sits at the clocks it
    # sustains (straight out of idle the first dozens of launches of a sub-millisecond kernel run 10-15 % slower).
    extra = {}
    if not args.no_extra:
        extra.update(extra_figures(B, synth, torch, dev))
        extra["calibration_step"] = calibration_step(B, torch, x, dy, theta, plan, y, codes, scales, quant, rows, n, heads,
                                                     bits, group, T)

    def step():
        B.bq_butterfly_fwd_quant(x, plan, codes, scales, quant, rows)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        step()
        b.record()
        events.append((a, b))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ts = [a.elapsed_time(b) for a, b in events]
    launch_ms = sum(ts) / len(ts)
    peaks.update(measured_fma(B, torch, dev))

    itemsize = 2
    bpr = alg_bytes_per_row("fwd_quant", n, heads, itemsize, bits, group, 2)
    fpr = alg_flops_per_row("fwd_quant", n, heads)
    gbs = bpr * T / (launch_ms * 1e-3) / 1e9
    tf = fpr * T / (launch_ms * 1e-3) / 1e12
    counters = {}
    cpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(cpath):
        try:
            counters = json.load(open(cpath))
        except Exception:
            counters = {}
    traffic = counters.get("fwd_quant_n4096_f16_int2_g128")
    valu_insts = counters.get("fwd_quant_n4096_f16_int2_g128_valu_wave_insts")  # SQ_INSTS_VALU of one launch
    issue = None
    if valu_insts:
        # one fp32 wave instruction occupies a SIMD for four cycles: the launch cannot be shorter than this at the
        # clock the FMA loop above ran at
        clock = peaks["fma_implied_clock_GHz"] * 1e9
        floor_ms = valu_insts * 4 / (SIMDS * clock) * 1e3
        issue = {"valu_wave_insts_per_launch": valu_insts, "per_thread_row": round(valu_insts * 64 / (T * 512), 1),
                 "issue_floor_ms": round(floor_ms, 4), "issue_frac": round(floor_ms / launch_ms, 4)}
    hbm_frac = gbs / HBM_PEAK_GBS
    alu_frac = tf / VALU_PEAK_TFLOPS
    alu_frac_unpacked = tf / VALU_PEAK_UNPACKED_TFLOPS
    # which roof binds: the one the launch is closer to, with the ALU roof taken as what this build can issue
    bound = "alu" if max(alu_frac_unpacked, issue["issue_frac"] if issue else 0.0) > hbm_frac else "hbm"
    roofline = {"kernel": "fused forward + INT2 quantisation, n=4096 fp16, group 128", "bound": bound,
                "launch_ms": round(launch_ms, 4), "launch_ms_min": round(min(ts), 4), "launch_ms_max": round(max(ts), 4),
                "traffic": traffic,
                "alg_bytes_per_launch": bpr * T, "alg_flops_per_launch": fpr * T}
    hbm = {"achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(hbm_frac, 4)}
    alu = {"achieved": round(tf, 2), "peak": VALU_PEAK_TFLOPS, "peak_published": VALU_PEAK_TFLOPS,
           "peak_unpacked": round(VALU_PEAK_UNPACKED_TFLOPS, 1), "unit": "TFLOP/s", "frac": round(alu_frac, 4),
           "frac_unpacked": round(alu_frac_unpacked, 4), "issue": issue}
    roofline.update(alu if bound == "alu" else hbm)
    roofline["hbm"] = hbm
    roofline["alu"] = alu

    if args.copy_ref:
        B.bq_probe_copy(x, y, x.numel() * x.element_size())
        torch.cuda.synchronize()
    out = {
        "metric": "rows/sec + achieved HBM GB/s (% peak), butterfly fwd+quant n=4096 fp16",
        "value": T / (ms_per_step * 1e-3),
        "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"calibration/prefill shape: n=4096, T={T} rows, fp16 Student-t(3) activations with "
                               "1% outlier channels x100; step = fused forward + INT2 quantisation (group 128, fp16 "
                               "scales), fp16 in, float32 arithmetic",
                   "n": n, "rows": T, "io_dtype": "f16", "bits": bits, "group": group},
        "fwd_quant_rows_per_s": T / (launch_ms * 1e-3),
        "fwd_quant_GBps": round(gbs, 1),
        "fwd_quant_hbm_frac": round(hbm_frac, 4),
        "roofline": roofline,
        "peaks": peaks,
    }
    out.update(extra)
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(args.cpu_rows)
    print(json.dumps(out))
    return 0


def calibration_step(B, torch, x, dy, theta, plan, y, codes, scales, quant, rows, n, heads, bits, group, T, steps=10):
    """The whole path on the same batch: plan build, fused forward + INT2 quantisation, forward, inverse, backward;
    every call timed with events, the sequence by the wall clock."""
    xi = torch.empty_like(x)
    dx = torch.empty_like(x)
    dtheta = torch.empty_like(theta)
    ws = torch.empty(max(256, B.bq_butterfly_bwd_workspace_bytes(rows)), dtype=torch.uint8, device=x.device)
    kernels = {
        "plan_build": lambda: B.bq_plan_build(theta, n, heads, plan),
        "fwd_quant": lambda: B.bq_butterfly_fwd_quant(x, plan, codes, scales, quant, rows),
        "fwd": lambda: B.bq_butterfly_fwd(x, y, plan, rows),
        "inv": lambda: B.bq_butterfly_inv(y, xi, plan, rows),
        "bwd": lambda: B.bq_butterfly_bwd(x, dy, plan, dx, dtheta, ws, rows),
    }
    order = ["plan_build", "fwd_quant", "fwd", "inv", "bwd"]
    for _ in range(3):
        for name in order:
            kernels[name]()
    torch.cuda.synchronize()
    events = {}
    t0 = time.perf_counter()
    for _ in range(steps):
        for name in order:
            a = torch.cuda.Event(enable_timing=True)
            b = torch.cuda.Event(enable_timing=True)
            a.record()
            kernels[name]()
            b.record()
            events.setdefault(name, []).append((a, b))
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms = (t1 - t0) * 1e3 / steps
    kinfo = {}
    for name in order:
        ts = [a.elapsed_time(b) for a, b in events[name]]
        avg = sum(ts) / len(ts)
        rec = {"avg_ms": round(avg, 4), "median_ms": round(sorted(ts)[len(ts) // 2], 4)}
        if name != "plan_build":
            bpr = alg_bytes_per_row(name, n, heads, 2, bits, group, 2)
            fpr = alg_flops_per_row(name, n, heads)
            gbs = bpr * T / (avg * 1e-3) / 1e9
            tf = fpr * T / (avg * 1e-3) / 1e12
            rec.update({"rows_per_s": T / (avg * 1e-3), "alg_bytes_per_row": bpr, "GBps": round(gbs, 1),
                        "hbm_frac": round(gbs / HBM_PEAK_GBS, 4), "alg_TFLOPps": round(tf, 2),
                        "valu_frac": round(tf / VALU_PEAK_TFLOPS, 4),
                        "valu_frac_unpacked": round(tf / VALU_PEAK_UNPACKED_TFLOPS, 4)})
        kinfo[name] = rec
    # each call once more on its own, 20 launches back to back: inside the sequence every kernel runs a few per cent
    # slower than alone (the five calls keep the device at its sustained limit)
    for name in order[1:]:
        avg, _, _ = time_kernel(kernels[name], 20, 10)
        kinfo[name]["alone_ms"] = round(avg, 4)
    kinfo["bwd"]["workspace_MiB"] = round(ws.numel() / 2 ** 20, 1)
    return {"workload": "plan build + fused fwd+INT2 quant + fwd + inv + bwd on the n=4096, T=%d fp16 batch" % T,
            "ms_per_step": round(ms, 4), "rows_per_s": T / (ms * 1e-3), "steps": steps, "kernels": kinfo}


def extra_figures(B, synth, torch, dev):
    """Figures for the other workload shapes (not part of the timed step)."""
    res = {}
    # decode latency: n=4096 fp16, T in {1, 8, 64}, fused forward + INT4, group 128
    wl = synth.make_workload(2, rows=64)
    theta = torch.from_numpy(wl.theta).to(dev)
    plan = B.alloc_plan(theta, wl.n, 1)
    xs = synth.storage_to_torch(wl.x, wl.dtype, dev)
    dec = {}
    cases = {}
    for T in (1, 8, 64):
        x = xs[:T].contiguous()
        codes, scales = B.alloc_quant_outputs(T, wl.n, 1, 4, 128, "f16", dev)
        cases[T] = (x, codes, scales, B.make_rows(x, wl.n, 1))
    q = B.make_quant(4, 128, "f16")
    samples = {T: [] for T in cases}
    for T, (x, codes, scales, rows) in cases.items():  # warm-up
        for _ in range(50):
            B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, rows)
    # per-call latency between two events; the batch sizes take turns (five rounds of 200 calls each), so that
    # whatever the device does between phases of the benchmark lands on all of them alike
    for _ in range(5):
        for T, (x, codes, scales, rows) in cases.items():
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
            for a, b in evs:
                a.record()
                B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, rows)
                b.record()
            torch.cuda.synchronize()
            samples[T] += [a.elapsed_time(b) for a, b in evs]
    for T, (x, codes, scales, rows) in cases.items():
        ts = samples[T]
        dec[f"T{T}"] = {"avg_us": round(sum(ts) / len(ts) * 1e3, 2), "median_us": round(percentile(ts, 0.5) * 1e3, 2),
                        "p99_us": round(percentile(ts, 0.99) * 1e3, 2), "max_us": round(max(ts) * 1e3, 2),
                        "calls": len(ts)}
        # 2000 calls back to back between two events (the events of the per-call figures cost about 2 us each)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(2000):
            B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, rows)
        e1.record()
        torch.cuda.synchronize()
        dec[f"T{T}"]["back_to_back_us"] = round(e0.elapsed_time(e1) / 2000 * 1e3, 2)
        # the same call 32 times in one HIP graph (the library only enqueues kernels, so it can be captured):
        # per-call time without the host's launch cost
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, rows)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(32):
                    B.bq_butterfly_fwd_quant(x, plan, codes, scales, q, rows)
        torch.cuda.synchronize()
        avg_g, med_g, _ = time_kernel(graph.replay, 30, 30)
        dec[f"T{T}"]["in_graph_us"] = round(med_g * 1e3 / 32, 2)
        del graph
    res["decode"] = {"workload": "n=4096 fp16 fused fwd+INT4 g128, event-timed per call on the stream (1000 calls per "
                                 "batch size, the sizes taking turns); back_to_back_us: 2000 calls between two events; "
                                 "in_graph_us: per call inside a captured graph of 32 calls", **dec}
    # per-head: 32 heads x n=128, T=8192, bf16, rotating over 6 buffers (> 256 MB in total)
    x4, th4, _ = synth.device_rows(4, 8192, dev)
    theta4 = torch.from_numpy(th4).to(dev)
    plan4 = B.alloc_plan(theta4, 128, 32)
    bufs = [x4] + [x4.clone() for _ in range(5)]
    codes4, scales4 = B.alloc_quant_outputs(8192, 128, 32, 4, 128, "f32", dev)
    rows4 = B.make_rows(x4, 128, 32)
    q4 = B.make_quant(4, 128, "f32")
    state = {"i": 0}

    def run4():
        state["i"] = (state["i"] + 1) % len(bufs)
        B.bq_butterfly_fwd_quant(bufs[state["i"]], plan4, codes4, scales4, q4, rows4)

    avg, med, mx = time_kernel(run4, 30, 30)
    bpr = alg_bytes_per_row("fwd_quant", 128, 32, 2, 4, 128, 4)
    res["per_head"] = {"workload": "32 heads x n=128, T=8192, bf16, fused fwd + per-head INT4",
                       "avg_ms": round(avg, 4), "rows_per_s": 8192 / (avg * 1e-3),
                       "GBps": round(bpr * 8192 / (avg * 1e-3) / 1e9, 1),
                       "hbm_frac": round(bpr * 8192 / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    # the backward pass on the same shape (everything in registers, no LDS)
    dy4 = bufs[1]
    dx4 = torch.empty_like(x4)
    dth4 = torch.empty_like(theta4)
    ws4 = torch.empty(max(256, B.bq_butterfly_bwd_workspace_bytes(rows4)), dtype=torch.uint8, device=dev)
    avg, med, mx = time_kernel(lambda: B.bq_butterfly_bwd(x4, dy4, plan4, dx4, dth4, ws4, rows4), 30, 30)
    bprb = alg_bytes_per_row("bwd", 128, 32, 2)
    res["per_head_bwd"] = {"workload": "32 heads x n=128, T=8192, bf16: dx and dtheta", "avg_ms": round(avg, 4),
                           "rows_per_s": 8192 / (avg * 1e-3), "GBps": round(bprb * 8192 / (avg * 1e-3) / 1e9, 1),
                           "hbm_frac": round(bprb * 8192 / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    del bufs, x4, dy4, dx4, ws4
    # backward at n=8192, T=65536, bf16
    T5 = 65536
    x5, th5, dy5 = synth.device_rows(5, T5, dev, want_dy=True)
    theta5 = torch.from_numpy(th5).to(dev)
    plan5 = B.alloc_plan(theta5, 8192, 1)
    dx5 = torch.empty_like(x5)
    dth5 = torch.empty_like(theta5)
    rows5 = B.make_rows(x5, 8192, 1)
    ws5 = torch.empty(max(256, B.bq_butterfly_bwd_workspace_bytes(rows5)), dtype=torch.uint8, device=dev)
    avg, med, mx = time_kernel(lambda: B.bq_butterfly_bwd(x5, dy5, plan5, dx5, dth5, ws5, rows5), 20, 15)
    bpr = alg_bytes_per_row("bwd", 8192, 1, 2)
    fpr = alg_flops_per_row("bwd", 8192, 1)
    res["bwd_n8192"] = {"workload": "n=8192, T=65536, bf16: dx and dtheta", "avg_ms": round(avg, 4),
                        "rows_per_s": T5 / (avg * 1e-3), "GBps": round(bpr * T5 / (avg * 1e-3) / 1e9, 1),
                        "hbm_frac": round(bpr * T5 / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                        "alg_TFLOPps": round(fpr * T5 / (avg * 1e-3) / 1e12, 2),
                        "valu_frac": round(fpr * T5 / (avg * 1e-3) / 1e12 / VALU_PEAK_TFLOPS, 4)}
    # forward kernels at n=8192 on the same rows (1024-thread workgroups, layer 13 across the halves in LDS)
    y5 = dx5
    c5, s5 = B.alloc_quant_outputs(T5, 8192, 1, 2, 128, "f16", dev)
    q5 = B.make_quant(2, 128, "f16")
    a_f, _, _ = time_kernel(lambda: B.bq_butterfly_fwd(x5, y5, plan5, rows5), 30, 30)
    a_i, _, _ = time_kernel(lambda: B.bq_butterfly_inv(x5, y5, plan5, rows5), 30, 30)
    a_q, _, _ = time_kernel(lambda: B.bq_butterfly_fwd_quant(x5, plan5, c5, s5, q5, rows5), 30, 30)
    b_f = alg_bytes_per_row("fwd", 8192, 1, 2)
    b_q = alg_bytes_per_row("fwd_quant", 8192, 1, 2, 2, 128, 2)
    res["fwd_n8192"] = {"workload": "n=8192, T=65536, bf16: forward, inverse, fused forward + INT2 g128",
                        "fwd_ms": round(a_f, 4), "fwd_GBps": round(b_f * T5 / (a_f * 1e-3) / 1e9, 1),
                        "inv_ms": round(a_i, 4), "inv_GBps": round(b_f * T5 / (a_i * 1e-3) / 1e9, 1),
                        "fwd_quant_ms": round(a_q, 4), "fwd_quant_GBps": round(b_q * T5 / (a_q * 1e-3) / 1e9, 1)}
    del x5, dy5, dx5, y5, ws5, c5, s5
    # fake-quantised forward (Dequant(Quant(Bx)) + code-bin histogram) on the calibration batch, INT2 g128
    T3 = 262144
    x3, th3, _ = synth.device_rows(3, T3, dev)
    theta3 = torch.from_numpy(th3).to(dev)
    plan3 = B.alloc_plan(theta3, 4096, 1)
    rows3 = B.make_rows(x3, 4096, 1)
    yq3 = torch.empty_like(x3)
    hist3 = torch.zeros(4, dtype=torch.int64, device=dev)
    q3 = B.make_quant(2, 128, "f16")
    avg, med, mx = time_kernel(lambda: B.bq_butterfly_fwd_fakequant(x3, plan3, yq3, hist3, q3, rows3), 30, 30)
    bpr = alg_bytes_per_row("fwd", 4096, 1, 2)
    res["fakequant"] = {"workload": "n=4096, T=262144, fp16: Dequant(Quant(Bx)) INT2 g128 + bin histogram",
                        "avg_ms": round(avg, 4), "rows_per_s": T3 / (avg * 1e-3),
                        "GBps": round(bpr * T3 / (avg * 1e-3) / 1e9, 1),
                        "hbm_frac": round(bpr * T3 / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    # the fused kernel with INT4 codes on the same batch
    c34, s34 = B.alloc_quant_outputs(T3, 4096, 1, 4, 128, "f16", dev)
    q34 = B.make_quant(4, 128, "f16")
    avg, med, mx = time_kernel(lambda: B.bq_butterfly_fwd_quant(x3, plan3, c34, s34, q34, rows3), 30, 30)
    bpr4 = alg_bytes_per_row("fwd_quant", 4096, 1, 2, 4, 128, 2)
    res["fwd_quant_int4"] = {"workload": "n=4096, T=262144, fp16: fused forward + INT4 g128, fp16 scales",
                             "avg_ms": round(avg, 4), "rows_per_s": T3 / (avg * 1e-3),
                             "GBps": round(bpr4 * T3 / (avg * 1e-3) / 1e9, 1),
                             "hbm_frac": round(bpr4 * T3 / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    del c34, s34
    # float32 rows (the 1e-5 tolerance class) at the same width: half the rows, the same bytes
    Tf = T3 // 2
    xf = x3[:Tf].float()
    yf = torch.empty_like(xf)
    rf = B.make_rows(xf, 4096, 1)
    cf, sf = B.alloc_quant_outputs(Tf, 4096, 1, 2, 128, "f16", dev)
    a_f, _, _ = time_kernel(lambda: B.bq_butterfly_fwd(xf, yf, plan3, rf), 30, 30)
    a_i, _, _ = time_kernel(lambda: B.bq_butterfly_inv(xf, yf, plan3, rf), 30, 30)
    a_q, _, _ = time_kernel(lambda: B.bq_butterfly_fwd_quant(xf, plan3, cf, sf, q3, rf), 30, 30)
    b_f = alg_bytes_per_row("fwd", 4096, 1, 4)
    b_q = alg_bytes_per_row("fwd_quant", 4096, 1, 4, 2, 128, 2)
    res["f32_rows"] = {"workload": "n=4096, T=131072, float32 rows: forward, inverse, fused forward + INT2 g128",
                       "fwd_ms": round(a_f, 4), "fwd_GBps": round(b_f * Tf / (a_f * 1e-3) / 1e9, 1),
                       "inv_ms": round(a_i, 4), "inv_GBps": round(b_f * Tf / (a_i * 1e-3) / 1e9, 1),
                       "fwd_quant_ms": round(a_q, 4), "fwd_quant_GBps": round(b_q * Tf / (a_q * 1e-3) / 1e9, 1),
                       "fwd_quant_hbm_frac": round(b_q * Tf / (a_q * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    del xf, yf, cf, sf
    # The fixed Hadamard rotation as baseline (paper, "Inference Efficiency": the learned transform's overhead over
    # the fast Hadamard transform): the add/sub kernel (no plan, no coefficient registers, one scale) against the
    # butterfly kernel with learned angles on the same batch, and the butterfly kernel with every angle at pi/4.
    import math
    y3 = yq3
    a_rand, _, _ = time_kernel(lambda: B.bq_butterfly_fwd(x3, y3, plan3, rows3), 30, 30)
    a_fht, _, _ = time_kernel(lambda: B.bq_hadamard_fwd(x3, y3, rows3), 30, 30)
    plan_h = B.alloc_plan(torch.full_like(theta3, math.pi / 4), 4096, 1)
    a_had, _, _ = time_kernel(lambda: B.bq_butterfly_fwd(x3, y3, plan_h, rows3), 30, 30)
    b_f = alg_bytes_per_row("fwd", 4096, 1, 2)
    res["hadamard_baseline"] = {"workload": "n=4096, T=262144, fp16 forward: learned butterfly vs add/sub Hadamard "
                                            "kernel (bq_hadamard_fwd) vs butterfly kernel with all angles pi/4",
                                "butterfly_ms": round(a_rand, 4), "fht_ms": round(a_fht, 4),
                                "butterfly_at_quarter_pi_ms": round(a_had, 4),
                                "butterfly_over_fht": round(a_rand / a_fht, 4),
                                "fht_GBps": round(b_f * T3 / (a_fht * 1e-3) / 1e9, 1),
                                "butterfly_GBps": round(b_f * T3 / (a_rand * 1e-3) / 1e9, 1)}
    del yq3, y3
    # composite transform for a width that is not a power of two: 5120 = 40 x 128, fp16
    Tk, d1k, d2k = 65536, 40, 128
    xk = x3.reshape(-1)[: Tk * d1k * d2k].view(Tk, d1k * d2k)
    yk = torch.empty_like(xk)
    thk = (torch.rand(1, 7, 64, device=dev) * 2 - 1) * math.pi
    plank = B.alloc_plan(thk, d2k, 1)
    q1 = torch.empty(d1k, d1k, dtype=torch.float32, device=dev)
    B.bq_cayley_build(torch.randn(d1k * (d1k - 1) // 2, device=dev) * 0.3, d1k, q1)
    rk = B.make_kron_rows(xk, d2k)
    avg, med, mx = time_kernel(lambda: B.bq_kron_fwd(xk, yk, q1, d1k, plank, rk), 30, 30)
    bprk = 2 * d1k * d2k * 2
    res["kron_5120"] = {"workload": "d = 5120 = 40 x 128, T=65536, fp16: (Cayley 40x40) (x) (butterfly 128)",
                        "avg_ms": round(avg, 4), "rows_per_s": Tk / (avg * 1e-3),
                        "GBps": round(bprk * Tk / (avg * 1e-3) / 1e9, 1),
                        "hbm_frac": round(bprk * Tk / (avg * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                        "mfma_TFLOPps": round(2 * d1k * d1k * d2k * Tk / (avg * 1e-3) / 1e12, 2)}
    del yk
    # weight side: W [11008, 4096] fp16 -> W B^T, group-wise INT2 (g128) and its dtheta contribution
    m = 11008
    Wt = x3[:m]
    dWt = x3[m:2 * m]
    rw = B.make_rows(Wt, 4096, 1)
    cw, sw = B.alloc_quant_outputs(m, 4096, 1, 2, 128, "f16", dev)
    dthw = torch.empty_like(theta3)
    wsw = torch.empty(max(256, B.bq_butterfly_bwd_workspace_bytes(rw)), dtype=torch.uint8, device=dev)
    a1, _, _ = time_kernel(lambda: B.bq_butterfly_fwd_quant(Wt, plan3, cw, sw, q3, rw), 30, 30)
    a2, _, _ = time_kernel(lambda: B.bq_butterfly_bwd(Wt, dWt, plan3, None, dthw, wsw, rw), 30, 30)
    res["weight_side"] = {"workload": "W [11008, 4096] fp16: fused W B^T + INT2 g128; dtheta from (W, dL/dW')",
                          "fwd_quant_ms": round(a1, 4), "bwd_ms": round(a2, 4)}
    del Wt, dWt, cw, sw, wsw
    # the method end to end on synthetic data: SGD with a cosine schedule from the identity on one linear layer
    # (paper, "Implementation Details"), W2A4, every butterfly call in the library, the layer's two dense
    # products in torch
    from paper_2509_09679_amd.calibration import ButterflyCalibrator, QuantSpec

    Tc, mc = 16384, 4096
    Xc, _, _ = synth.device_rows(3, Tc, dev)
    g = torch.Generator(device=dev).manual_seed(7)
    Wc = (torch.randn((mc, 4096), generator=g, device=dev) * 0.02).to(Xc.dtype)
    cal = ButterflyCalibrator(Wc, QuantSpec(4, 128, "f16"), QuantSpec(2, 128, "f16"))
    cal.fit(Xc, 2, 1.0)  # warm-up
    cal.theta.zero_()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    losses = cal.fit(Xc, 30, 1.0)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    res["calibration_fit"] = {"workload": "30 SGD steps from theta = 0 on one layer: X [16384, 4096] fp16 (INT4 g128), "
                                          "W [4096, 4096] fp16 (INT2 g128); loss = L_recon, L_uniform reported",
                              "ms_per_step": round((t1 - t0) * 1e3 / 30, 3), "loss_first": losses[0], "loss_last": losses[-1],
                              "loss_min": min(losses), "L_uniform_first": round(cal.kl_seen[0], 5),
                              "L_uniform_last": round(cal.kl_seen[-1], 5)}
    return res


if __name__ == "__main__":
    sys.exit(main())
