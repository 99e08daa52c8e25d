#!/usr/bin/env python3
"""Throughput of the GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

One step = one gemm_run over one batch of synthetic input (seeded, generated on
the host, resident in HBM before the timed region).  Prints ONE JSON line with
the throughput (TFLOP/s for matrix-core-bound shapes, GB/s for HBM-bound ones),
the roofline fraction of the kernel measured with HIP events on the launch
stream, and the CPU oracle timed on a bounded sample of the same workload.

The timing follows the paper's protocol (App. "Benchmarking kernel runtime"):
an untimed warm-up of at least --warmup launches, one second and ten launches,
then exactly --steps launches between two synchronisations (median / min / p10 /
p90 of single launches come from a following pass with an event per launch), and
no result is cached or reused between launches (HBM-bound
shapes rotate through several weight buffers so that the last-level cache cannot
serve them).  Shader clock and board power are sampled from sysfs while the
warm-up and the timed launches run.  The default line also carries a `secondary`
entry: the decode-shaped GEMV (M = 1, N = K = 8192) measured the same way.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

PEAK_MFMA_TFLOPS = 2516.6     # dense bf16/fp16: 256 CU x 4096 FLOP/clk x 2.4 GHz
PEAK_MFMA_F8_TFLOPS = 5033.2  # dense fp8: twice that
PEAK_HBM_GBS = 8000.0
PEAK_FP32_TFLOPS = 157.3


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--splitk", type=int, default=None,
                    help="plan the product as split-K with this many K slices (0 = built-in choice); "
                         "the workspace is allocated once, outside the timed region")
    ap.add_argument("--workload", default="square_8192", choices=sorted(wl.WORKLOADS) + sorted(wl.ROPE_WORKLOADS))
    ap.add_argument("--config", default=None, help="tile configuration name (default: built-in choice)")
    ap.add_argument("--tune", action="store_true",
                    help="pick the tile configuration with gemm_tune (times every applicable one first)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the second headline shape (M = 1, N = K = 8192) that the default line also carries")
    ap.add_argument("--no-measured-peak", action="store_true",
                    help="skip the MFMA-only / streaming-read probe that the roofline fraction is also related to")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (for scaling HBM byte counters under a profiler)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def source_hash(files=None):
    """Hash of kernel sources (`files`: names under csrc/, default all of them): counter readings taken
    for another version of a kernel do not count."""
    import glob
    import hashlib
    csrc = os.path.join(ROOT, "paper_2603_12440_amd", "csrc")
    paths = sorted(glob.glob(os.path.join(csrc, "*"))) if files is None else [os.path.join(csrc, f) for f in sorted(files)]
    h = hashlib.sha256()
    for f in paths:
        if not os.path.exists(f):
            return None
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per launch (fetch + write) from the committed rocprofv3 counter summary, or None if
    there is none for this workload and this version of its kernel (a line names the source files
    the kernel is compiled from and carries their hash at the time the counters were read)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 6 and not line.startswith("#") and f[0] == workload and f[2] == source_hash(f[5].split(",")):
            return float(f[3]) + float(f[4])
    return None


def gpu_desc(g, w):
    dt = {"f32": g.F32, "bf16": g.BF16, "f16": g.F16, "f8": g.F8E4M3}
    lay = {"row": g.ROW_MAJOR, "col": g.COL_MAJOR}
    return g.GemmDesc(w.M, w.N, w.K, dtype=dt[w.dtype], dtype_c=dt[w.out_dtype or w.dtype],
                      layout_a=lay[w.layout_a], layout_b=lay[w.layout_b],
                      epilogue=g.EPILOGUES[w.epilogue], batch=w.batch, scale=w.scale)


def cpu_baseline(w, A, B, bias, target_s, gpu_out):
    """The CPU leg: time the oracle (as it stands) on a bounded sample (the first R
    rows of the output, all N columns, full K; R from a small calibration run), and
    check sampled entries of the GPU result of the last timed launch against it."""
    import oracle
    oracle.build()
    dt = {"f32": oracle.DTYPE_F32, "bf16": oracle.DTYPE_BF16, "f16": oracle.DTYPE_F16, "f8": oracle.DTYPE_F8E4M3}
    lay = {"row": oracle.ROW_MAJOR, "col": oracle.COL_MAJOR}
    epi = {"none": oracle.EPI_NONE, "bias": oracle.EPI_BIAS, "bias_relu": oracle.EPI_BIAS_RELU,
           "bias_gelu_erf": oracle.EPI_BIAS_GELU_ERF, "bias_gelu_tanh": oracle.EPI_BIAS_GELU_TANH,
           "relu": oracle.EPI_RELU, "gelu_erf": oracle.EPI_GELU_ERF,
           "bias_swish_scale": oracle.EPI_BIAS_SWISH_SCALE,
           "bias_sigmoid_scale_residual": oracle.EPI_BIAS_SIGMOID_SCALE_RESIDUAL,
           "swish_scale": oracle.EPI_SWISH_SCALE,
           "sigmoid_scale_residual": oracle.EPI_SIGMOID_SCALE_RESIDUAL}

    def oracle_problem(o, x):
        return o.Problem(x.M, x.N, x.K, dt[x.dtype], dt[x.dtype], lay[x.layout_a], lay[x.layout_b],
                         epilogue=epi[x.epilogue], batch=x.batch, scale=x.scale)

    a, b = wl.storage_numpy(A), wl.storage_numpy(B)
    bz = None if bias is None else bias.numpy()

    # sampled check of the GPU output: |C - y| within K u S (any-order fp32 accumulation of
    # exact products) + epilogue slack + one rounding to the output type
    pb, pi, pj = wl.sample_points(w, 2048, 99)
    ref = oracle.ref_gemm_points(oracle_problem(oracle, w), a, b, bz, pb, pi, pj, want=("y", "t", "s"))
    got = gpu_out.to(torch.float64).numpy()[pb, pi, pj]
    u_out = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -24}[w.out_dtype or w.dtype]
    acc = 1.13 * w.K * 2.0 ** -24 * ref["s"] + 16 * 2.0 ** -24 * (np.abs(ref["t"]) + 1.0)
    bound = acc + u_out * (np.abs(ref["y"]) + acc) * 1.001 + 1e-30
    matches = bool(np.all(np.abs(got - ref["y"]) <= bound))

    def run(rows):
        sub = wl.scaled(w, M=rows, batch=1)
        p = oracle_problem(oracle, sub)
        t0 = time.perf_counter()
        run.last = oracle.ref_gemm(p, a, b, bz, want=("y",))
        return time.perf_counter() - t0

    cores = oracle.num_threads()
    r0 = min(w.M, max(1, cores))
    t_cal = run(r0)
    per_row = max(t_cal / r0, 1e-9)
    rows = int(min(w.M, max(r0, target_s / per_row)))
    rows = max(cores, rows - rows % cores) if rows >= cores else rows
    t = run(rows)
    # every element of the rows just computed against the GPU's: the same bound with S replaced by
    # its Cauchy-Schwarz majorant |a_i| |b_j| (the timed call returns y only)
    if w.epilogue == "none":
        af = wl.to_float64(A[0, :rows] if w.layout_a == "row" else A[0, :, :rows].T)
        bf = wl.to_float64(B[0] if w.layout_b == "col" else B[0].T)
        na, nb = np.sqrt((af * af).sum(axis=1)), np.sqrt((bf * bf).sum(axis=1))
        yr = run.last["y"].reshape(rows, w.N)
        gr = gpu_out[0, :rows].to(torch.float64).numpy()
        accr = 1.13 * w.K * 2.0 ** -24 * np.outer(na, nb)
        rows_ok = bool(np.all(np.abs(gr - yr) <= accr + u_out * (np.abs(yr) + accr) * 1.001 + 1e-30))
        matches = matches and rows_ok
        rows_note = f"; all {rows} x {w.N} of these outputs compared with the GPU's: {'ok' if rows_ok else 'MISMATCH'}"
    else:
        rows_note = ""
    flops = 2.0 * rows * w.N * w.K
    if w.bound == "hbm":
        e = 2 if w.dtype != "f32" else 4
        val, unit = e * (rows * w.K + w.K * w.N + rows * w.N) / t / 1e9, "GB/s"
    else:
        val, unit = flops / t / 1e12, "TFLOP/s"
    return {"value": val, "unit": unit, "cores": cores, "kind": "oracle",
            "gpu_output_matches_oracle_samples": matches,
            "sample": f"first {rows} of {w.M} output rows x all {w.N} columns, full K={w.K}, "
                      f"batch 0, fp64 triple loop, {t:.2f} s wall" + rows_note}


def measured_peak(g, dev, bound, dtype):
    """What the hardware delivers when it does nothing else (include/probe.h): an MFMA-only register
    loop for the matrix-core bound, a streaming read of 1.25 GiB for the HBM bound.  None for the
    other bounds."""
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    if bound == "mfma" and dtype in ("bf16", "f16", "f8"):
        code = {"f16": g.F16, "f8": g.F8E4M3}.get(dtype, g.BF16)
        out = {"value": round(g.probe_mfma_peak(code, sink, min_seconds=0.3), 1), "unit": "TFLOP/s",
               "what": ("v_mfma_f32_32x32x64_f8f6f4" if dtype == "f8" else "v_mfma_f32_32x32x16") +
                       " register loop, 8 waves per CU, fixed pseudo-random operands",
               "value_fresh_operands": round(g.probe_mfma_peak(code, sink, min_seconds=0.3, refresh_operands=True), 1)}
        if dtype != "f8":            # the shape the default 16-bit kernel multiplies with
            out["v_mfma_f32_16x16x32"] = {
                "value": round(g.probe_mfma16_peak(code, sink, min_seconds=0.3), 1),
                "value_fresh_operands": round(g.probe_mfma16_peak(code, sink, min_seconds=0.3, refresh_operands=True), 1)}
        return out
    if bound == "hbm":
        n = 5 << 28
        buf = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
        out = {"value": round(g.probe_read_peak(buf, n, sink, min_seconds=0.3), 1), "unit": "GB/s",
               "what": "streaming read of 1.25 GiB, 16 KB per wave, non-temporal"}
        del buf
        return out
    return None


def copy_calibration(dev):
    """A plain device copy of known size (reads 1 GiB, writes 1 GiB): the yardstick the byte
    counters of a profiler run are scaled by."""
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


class Telemetry:
    """Samples the shader clock (the starred level of pp_dpm_sclk) and the board power (hwmon
    power1_input, microwatts) of card0 from sysfs in a background thread."""

    def __init__(self, period=0.01):
        import glob
        self.period = period
        self.sclk_path = next(iter(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")), None)
        self.power_path = next(iter(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input")), None) or \
            next(iter(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_average")), None)
        self.sclk, self.power = [], []
        self._stop = False
        self._thread = None

    def _read(self):
        try:
            if self.sclk_path:
                for line in open(self.sclk_path):
                    if "*" in line:
                        self.sclk.append(float(line.split(":")[1].lower().replace("mhz", "").replace("*", "").strip()))
            if self.power_path:
                self.power.append(float(open(self.power_path).read()) * 1e-6)
        except (OSError, ValueError, IndexError):
            pass

    def __enter__(self):
        import threading

        def loop():
            while not self._stop:
                self._read()
                time.sleep(self.period)
        self._thread = threading.Thread(target=loop, daemon=True)
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop = True
        self._thread.join()

    def summary(self):
        def med(v):
            return round(float(np.median(v)), 1) if v else None
        return {"sclk_mhz_median": med(self.sclk), "sclk_mhz_min": round(min(self.sclk), 1) if self.sclk else None,
                "power_w_median": med(self.power), "power_w_max": round(max(self.power), 1) if self.power else None,
                "samples": max(len(self.sclk), len(self.power)),
                "what": "sysfs pp_dpm_sclk / hwmon power1, sampled while the warm-up and the timed launches ran"}


def timed_launches(step, steps, warmup, min_warm_seconds=1.0, min_warm_launches=10):
    """The paper's protocol around `step(i)`: untimed warm-up (at least `warmup` launches, and until
    `min_warm_seconds` and `min_warm_launches` have passed), then exactly `steps` launches between two
    synchronisations (one event before, one after).  Returns (wall ms per step, mean kernel ms per step
    from the two events, per-launch statistics from a following pass, launches of the warm-up)."""
    n = 0
    t0 = time.perf_counter()
    while n < warmup or n < min_warm_launches or time.perf_counter() - t0 < min_warm_seconds:
        for _ in range(8):
            step(n)
            n += 1
        torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        step(n + i)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = ev0.elapsed_time(ev1) / steps
    # the spread of single launches, in a pass of its own (an event between launches costs a
    # microsecond or two of idle time each, which the mean above should not carry)
    m = min(steps, 200)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(m + 1)]
    ev[0].record()
    for i in range(m):
        step(n + steps + i)
        ev[i + 1].record()
    torch.cuda.synchronize()
    per = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(m)])
    stats = {"median_ms": round(float(np.median(per)), 6), "min_ms": round(float(per.min()), 6),
             "p10_ms": round(float(np.percentile(per, 10)), 6), "p90_ms": round(float(np.percentile(per, 90)), 6),
             "launches": m,
             "what": "durations between consecutive events, one event per launch, in a pass after the timed region"}
    return wall * 1e3 / steps, kern_ms, stats, n


def bench_secondary(g, dev, name="skinny_m1_n8192", steps=400):
    """The second headline shape, measured like the first: the decode-shaped GEMV with rotated weight
    buffers, its roofline fraction, and every output checked against the oracle."""
    w = wl.WORKLOADS[name]
    A, B, bias = wl.make_inputs(w)
    plan = g.gemm_create(gpu_desc(g, w))
    nbuf = min(64, max(2, int(np.ceil(1.2e9 / w.bytes))))
    Ad = [A.to(dev) for _ in range(nbuf)]
    Bd = [B.to(dev) for _ in range(nbuf)]
    Cd = [torch.empty((w.batch, w.M, w.N), dtype=wl.TORCH_DTYPE[w.out_dtype or w.dtype], device=dev) for _ in range(nbuf)]
    stream = torch.cuda.current_stream().cuda_stream

    def step(i):
        j = i % nbuf
        g.gemm_run(plan, Ad[j], Bd[j], Cd[j], None, stream)
    ms_wall, ms_kern, stats, _ = timed_launches(step, steps, 20, min_warm_seconds=0.3)
    info = plan.info()
    g.gemm_destroy(plan)
    achieved = w.bytes / (ms_kern * 1e-3) / 1e9
    import oracle
    oracle.build()
    p = oracle.Problem(w.M, w.N, w.K, oracle.DTYPE_BF16, oracle.DTYPE_BF16, oracle.ROW_MAJOR, oracle.COL_MAJOR)
    ref = oracle.ref_gemm(p, wl.storage_numpy(A), wl.storage_numpy(B), None, want=("y", "s"))
    got = Cd[0].to(torch.float64).cpu().numpy().reshape(ref["y"].shape)
    acc = w.K * 2.0 ** -24 * ref["s"]
    ok = bool(np.all(np.abs(got - ref["y"]) <= acc + 2.0 ** -8 * (np.abs(ref["y"]) + acc) * 1.001 + 1e-30))
    return {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "metric": "HBM-bound GEMM throughput (algorithmic bytes / time)",
            "value": round(w.bytes / (ms_wall * 1e-3) / 1e9, 3), "unit": "GB/s", "steps": steps,
            "ms_per_step": round(ms_wall, 6), "per_launch": stats, "plan": info, "buffers_rotated": nbuf,
            "roofline": {"bound": "hbm", "achieved": round(achieved, 3), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": measured_traffic(w.name)},
            "gpu_output_matches_oracle": ok, "oracle_check": f"all {w.M * w.N} outputs, fp64 oracle, a-priori bound"}, ok


def bench_rope(args, g, dev):
    """A rotary-embedding workload: one step = the query and the key tensor of a layer rotated in
    one launch (include/rope.h).  HBM-bound: algorithmic bytes = every element read and written once."""
    w = wl.ROPE_WORKLOADS[args.workload]
    q, k, cos, sin = wl.make_rope_inputs(w)
    gd = {"f32": g.F32, "bf16": g.BF16, "f16": g.F16}
    desc = g.RopeDesc(w.batch, w.seq, w.head_dim, dtype=gd[w.dtype], table_dtype=gd[w.table_dtype])
    nbuf = min(64, max(2, int(np.ceil(1.2e9 / w.bytes))))          # no reuse out of the last-level cache
    qd, kd = [q.to(dev) for _ in range(nbuf)], [k.to(dev) for _ in range(nbuf)]
    qy, ky = [torch.empty_like(t) for t in qd], [torch.empty_like(t) for t in kd]
    cosd, sind = cos.to(dev), sin.to(dev)
    stream = torch.cuda.current_stream().cuda_stream

    def tensor(x, y, heads):
        st = (w.seq * heads * w.head_dim, w.head_dim, heads * w.head_dim)     # [b, s, h, d] memory
        return g.RopeTensor(x, y, heads, st, st)
    sets = [[tensor(qd[j], qy[j], w.heads_q), tensor(kd[j], ky[j], w.heads_k)] for j in range(nbuf)]

    def step(i):
        g.rope_apply(desc, sets[i % nbuf], cosd, sind, stream)

    if args.copy_calibration:
        copy_calibration(dev)

    with Telemetry() as tel:
        ms_per_step, kern_ms, per_launch, warm_launches = timed_launches(step, args.steps, args.warmup)
    last_step = warm_launches + args.steps - 1
    achieved = w.bytes / (kern_ms * 1e-3) / 1e9
    out = {
        "metric": "rotary embedding throughput (algorithmic bytes / time)",
        "value": round(w.bytes / (ms_per_step * 1e-3) / 1e9, 3), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "per_launch": per_launch, "warmup_launches_run": warm_launches, "telemetry": tel.summary(),
        "config": {"workload": w.name, "batch": w.batch, "heads_q": w.heads_q, "heads_k": w.heads_k,
                   "seq": w.seq, "head_dim": w.head_dim, "storage": w.dtype, "tables": w.table_dtype,
                   "layout": "[batch, seq, heads, head_dim] memory, rotated as [batch, heads, seq, head_dim]",
                   "buffers_rotated": nbuf},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 3), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": measured_traffic(w.name)},
    }
    if not args.no_measured_peak and not args.copy_calibration:
        mp = measured_peak(g, dev, "hbm", w.dtype)
        out["roofline"]["measured_peak"] = mp
        out["roofline"]["frac_of_measured"] = round(achieved / mp["value"], 4)
    ok = True
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        od = {"f32": oracle.DTYPE_F32, "bf16": oracle.DTYPE_BF16, "f16": oracle.DTYPE_F16}
        # the oracle on a bounded sample: the first P positions of every batch, both tensors
        per_pos = w.batch * (w.heads_q + w.heads_k) * w.head_dim
        P = 8
        t_cal = None
        for _ in range(2):
            P = min(w.seq, P)
            t0 = time.perf_counter()
            refs = []
            for x, heads in ((q, w.heads_q), (k, w.heads_k)):
                xs = x[:, :P].contiguous()
                refs.append(oracle.ref_rope(w.batch, heads, P, w.head_dim, wl.storage_numpy(xs),
                                            wl.storage_numpy(cos[:P].contiguous()), wl.storage_numpy(sin[:P].contiguous()),
                                            dtype_x=od[w.dtype], dtype_table=od[w.table_dtype],
                                            stride_b=P * heads * w.head_dim, stride_h=w.head_dim,
                                            stride_s=heads * w.head_dim))
            t = time.perf_counter() - t0
            if t_cal is None and P < w.seq:
                t_cal = t
                P = int(max(P, min(w.seq, P * args.cpu_seconds / max(t, 1e-6))))
                continue
            break
        j = last_step % nbuf
        u = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -24}[w.dtype]
        for ref, y in zip(refs, (qy[j], ky[j])):
            got = wl.to_float64(y[:, :P].cpu().transpose(1, 2))
            ok = ok and bool(np.all(np.abs(got - ref) <= 1.01 * u * np.abs(ref) + 1e-5))
        e = 2 if w.dtype != "f32" else 4
        out["cpu_baseline"] = {"value": round(2 * e * P * per_pos / t / 1e9, 4), "unit": "GB/s", "cores": 1,
                               "kind": "oracle", "gpu_output_matches_oracle_samples": ok,
                               "sample": f"first {P} of {w.seq} positions of every batch, query and key "
                                         f"tensors, fp64 loop, {t:.2f} s wall"}
    print(json.dumps(out))
    return 0 if ok else 1


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only (the library has no multi-GPU path); run with --gpus 1",
              file=sys.stderr)
        return 2
    import paper_2603_12440_amd as g
    g.load_library()                      # raises if the HIP library is missing
    if not torch.cuda.is_available():
        raise RuntimeError("no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.workload in wl.ROPE_WORKLOADS:
        return bench_rope(args, g, dev)
    w = wl.WORKLOADS[args.workload]
    A, B, bias = wl.make_inputs(w)
    desc = gpu_desc(g, w)
    cfg = -1 if args.config is None else g.config_names().index(args.config)
    if args.tune:
        odt0 = wl.TORCH_DTYPE[w.out_dtype or w.dtype]            # the descriptor's dtype_c: every candidate writes that
        c_tune = torch.empty((w.batch, w.M, w.N), dtype=odt0, device=dev)
        assert c_tune.numel() * c_tune.element_size() == w.batch * w.M * w.N * {"f32": 4, "bf16": 2, "f16": 2}[w.out_dtype or w.dtype]
        cfg, _ = g.gemm_tune(desc, A.to(dev), B.to(dev), c_tune, None if bias is None else bias.to(dev), min_seconds=0.2)
        del c_tune
    plan = g.gemm_create_config(desc, cfg) if args.splitk is None else g.gemm_create_splitk(desc, args.splitk)
    info = plan.info()
    ws_bytes = g.gemm_workspace_bytes(plan)
    ws = torch.empty(max(ws_bytes, 16) // 4, dtype=torch.float32, device=dev) if ws_bytes else None

    # HBM-bound shapes: rotate through enough distinct copies of the operands that
    # the 256 MB last-level cache cannot hold them (no reuse between launches).
    nbuf = 1
    if w.bound == "hbm":
        nbuf = max(2, int(np.ceil(1.2e9 / w.bytes)))
        nbuf = min(nbuf, 64)
    Ad = [A.to(dev) for _ in range(nbuf)]
    Bd = [B.to(dev) for _ in range(nbuf)]
    odt = wl.TORCH_DTYPE[w.out_dtype or w.dtype]
    Cd = [torch.empty((w.batch, w.M, w.N), dtype=odt, device=dev) for _ in range(nbuf)]
    biasd = bias.to(dev) if bias is not None else None
    stream = torch.cuda.current_stream().cuda_stream

    def step(i):
        j = i % nbuf
        if ws is None:
            g.gemm_run(plan, Ad[j], Bd[j], Cd[j], biasd, stream)
        else:
            g.gemm_run_workspace(plan, Ad[j], Bd[j], Cd[j], biasd, ws, ws_bytes, stream)

    if args.copy_calibration:
        copy_calibration(dev)

    with Telemetry() as tel:
        ms_per_step, kern_ms, per_launch, warm_launches = timed_launches(step, args.steps, args.warmup)
    last_step = warm_launches + args.steps - 1           # (the buffers rotate with the launch count)

    if w.bound == "hbm":
        metric, unit = "HBM-bound GEMM throughput (algorithmic bytes / time)", "GB/s"
        value = w.bytes / (ms_per_step * 1e-3) / 1e9
        achieved, peak, bound, runit = w.bytes / (kern_ms * 1e-3) / 1e9, PEAK_HBM_GBS, "hbm", "GB/s"
    else:
        metric, unit = "GEMM throughput (2MNK / time)", "TFLOP/s"
        value = w.flops / (ms_per_step * 1e-3) / 1e12
        peak = {"f32": PEAK_FP32_TFLOPS, "f8": PEAK_MFMA_F8_TFLOPS}.get(w.dtype, PEAK_MFMA_TFLOPS)
        achieved, bound, runit = w.flops / (kern_ms * 1e-3) / 1e12, ("alu" if w.dtype == "f32" else "mfma"), "TFLOP/s"

    out = {
        "metric": metric, "value": round(value, 3), "unit": unit, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "per_launch": per_launch, "warmup_launches_run": warm_launches, "telemetry": tel.summary(),
        "config": {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "batch": w.batch,
                   "layout": f"A {w.layout_a}-major, B {w.layout_b}-major, C row-major",
                   "epilogue": w.epilogue, "plan": info, "buffers_rotated": nbuf},
        "roofline": {"bound": bound, "achieved": round(achieved, 3), "peak": peak, "unit": runit,
                     "frac": round(achieved / peak, 4), "traffic": measured_traffic(w.name)},
    }
    if not args.no_measured_peak and not args.copy_calibration:
        mp = measured_peak(g, dev, bound, w.dtype)
        if mp is not None:
            out["roofline"]["measured_peak"] = mp
            out["roofline"]["frac_of_measured"] = round(achieved / mp["value"], 4)
    ok = True
    if not args.no_cpu_baseline:
        # the paper's "no result reuse" rule: the last timed launch's output is checked
        last = Cd[last_step % nbuf].cpu()
        out["cpu_baseline"] = cpu_baseline(w, A, B, bias, args.cpu_seconds, last)
        ok = out["cpu_baseline"]["gpu_output_matches_oracle_samples"]
    g.gemm_destroy(plan)
    if args.workload == "square_8192" and not args.no_secondary and not args.copy_calibration:
        del Ad, Bd, Cd
        sec, sec_ok = bench_secondary(g, dev)
        out["secondary"] = [sec]
        ok = ok and sec_ok
    print(json.dumps(out))
    return 0 if ok else 1


if __name__ == "__main__":
    sys.exit(main())
