#!/usr/bin/env python3
"""Benchmark of the fused contraction hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--all]

A step is one call of the workload's entry point (pbk_matmul /
pbk_batched_matmul / pbk_conv2d_nhwc / pbk_attention) over seeded synthetic
inputs that are already resident in HBM.  Prints ONE JSON line: whole-job
TFLOP/s (2*M*N*K per step, epilogue flops not counted; 4*Nq*Nk*D per batch
entry for attention, softmax flops not counted), the roofline position of the kernel from HIP
event timings of every launch, and the CPU oracle timed on a bounded sample of
the same workload as a baseline.  --all adds a per-workload table on stderr (and,
with --json-out FILE, the same rows as JSON); the JSON line is always the
headline workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HEADLINE = "cfg2_bf16_8192"
PEAK_MFMA_16BIT_TFLOPS = 2516.6     # 256 CU x 4096 flop/clk/CU x 2.4 GHz (dense bf16/fp16)
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
DTYPE_NAMES = {0: "f32", 1: "bf16", 2: "f16", 3: "fp8_e4m3", 4: "fp8_e5m2", 5: "int8"}
PEAK_MFMA_FP8_TFLOPS = 5033.2       # twice the 16-bit rate
ROTATE_OVER_BYTES = 512 << 20       # twice the 256 MB memory-side cache


def is_attention(w):
    return hasattr(w, "Nq")


def is_int8(w):
    return type(w).__name__ == "Int8Workload"


def in_dtype_of(w):
    return 5 if is_int8(w) else w.dtype if is_attention(w) else w.in_dtype


def bound_of(w):
    """Which roofline bounds the workload: arithmetic intensity against the ridge."""
    import workloads as wl
    if is_int8(w):
        return ("mfma", PEAK_MFMA_FP8_TFLOPS)       # int8 dense MFMA: 5.0 POP/s, same rate as FP8
    if is_attention(w):
        peak = PEAK_FP32_TFLOPS if w.dtype == wl.DTYPE_F32 else PEAK_MFMA_16BIT_TFLOPS
        ridge = peak * 1e12 / (PEAK_HBM_GBS * 1e9)
        return ("mfma", peak) if w.flops / w.algorithmic_bytes >= ridge else ("hbm", PEAK_HBM_GBS)
    peak = (PEAK_FP32_TFLOPS if w.in_dtype == wl.DTYPE_F32 else
            PEAK_MFMA_FP8_TFLOPS if w.in_dtype in (wl.DTYPE_FP8_E4M3, wl.DTYPE_FP8_E5M2) else PEAK_MFMA_16BIT_TFLOPS)
    ridge = peak * 1e12 / (PEAK_HBM_GBS * 1e9)
    ai = w.flops / w.algorithmic_bytes
    return ("mfma", peak) if ai >= ridge else ("hbm", PEAK_HBM_GBS)


ZERO_OPERANDS = False      # set by --zero-operands


def time_workload(w, steps, warmup):
    """Returns dict with wall ms/step over the timed region and per-launch event times."""
    import torch
    import workloads as wl
    import pbk_testlib as T
    import paper_2603_06731_amd as pbk

    if is_int8(w):
        host = wl.make_int8_inputs(w)
        out = torch.empty(w.M * w.N, dtype=torch.int8, device="cuda")

        def run(w, dev, out=None, stream=None):
            return pbk.pbk_matmul_int8(dev["a"], dev["b"], out, w.M, w.N, w.K, w.K, w.K, w.N, 1, dev["scale"], dev["bias"],
                                       host["mid_scale"], dev["mul"], dev["add"], host["relu"], host["out_scale"],
                                       5, stream), out
        dev = {k: torch.from_numpy(v).cuda() for k, v in host.items() if hasattr(v, "dtype")}
    elif is_attention(w):
        host = wl.make_attention_inputs(w)
        out = T.device_empty(w.batch * w.Nq * w.D, w.dtype)
        run = T.run_attention
    else:
        host = wl.make_inputs(w)
        m, n, _ = w.gemm_mnk
        out = T.device_empty(w.batch * m * n, w.out_dtype)
        run = T.run_workload
    if not is_int8(w):
        dev = T.upload(host)
    if ZERO_OPERANDS:
        # power-limit probe: the same launches on all-zero A and B (the matrix units then draw far less power and
        # the chip holds its nominal clock); the figure says what the kernel sustains when the clock is not cut
        for key in ("a", "b", "q", "k", "v"):
            if key in dev and hasattr(dev[key], "zero_"):
                dev[key].zero_()
    # Working sets that fit the 256 MB memory-side cache are rotated over several copies of the inputs and
    # the output (enough to exceed twice that cache, at most 8), so that a launch does not find the operands
    # of the previous one still cached; larger ones need no rotation.
    set_bytes = sum(t.numel() * t.element_size() for t in dev.values() if hasattr(t, "numel")) + out.numel() * out.element_size()
    nsets = max(1, min(8, -(-ROTATE_OVER_BYTES // max(set_bytes, 1)))) if set_bytes < ROTATE_OVER_BYTES // 2 else 1
    sets = [(dev, out)] + [({k: (v.clone() if hasattr(v, "clone") else v) for k, v in dev.items()}, out.clone())
                           for _ in range(nsets - 1)]
    stream = torch.cuda.current_stream()
    for i in range(warmup):
        d, o = sets[i % nsets]
        st, _o = run(w, d, out=o, stream=stream)
        pbk.check(st, w.name)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        d, o = sets[i % nsets]
        starts[i].record(stream)
        st, _o = run(w, d, out=o, stream=stream)
        ends[i].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    pbk.check(st, w.name)
    ev_ms = [s.elapsed_time(e) for s, e in zip(starts, ends)]
    return {"wall_ms_per_step": (t1 - t0) * 1e3 / steps, "event_ms": ev_ms,
            "kernel": pbk.pbk_last_kernel(), "host": host, "out": out, "buffer_sets": nsets,
            "set_bytes": set_bytes}


def measure_copy_bandwidth(nbytes=1 << 30, reps=10):
    """Achievable HBM bandwidth in this run: a device copy of `nbytes` (read + write counted), and a fill
    (write only), timed with events."""
    import torch
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    src.fill_(1)
    res = {}
    for name, fn, moved in (("copy", lambda: dst.copy_(src), 2 * nbytes), ("fill", lambda: dst.fill_(2), nbytes)):
        for _ in range(2):
            fn()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = moved * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst
    return res


def cpu_baseline_attention(w, host, budget_s=15.0):
    """The attention oracle on a bounded number of query rows of the same workload."""
    import numpy as np
    import oracle
    threads = oracle.num_threads()

    def run(nrows):
        r = np.random.default_rng(3)
        sb = r.integers(0, w.batch, size=nrows)
        si = r.integers(0, w.Nq, size=nrows)
        t0 = time.perf_counter()
        if w.causal:
            oracle.attention_causal_rows(host["q"], host["k"], host["v"], sb, si, dtype=w.dtype, alpha=w.alpha)
        else:
            oracle.attention_rows(host["q"], host["k"], host["v"], host["bias"], sb, si, dtype=w.dtype, alpha=w.alpha)
        return time.perf_counter() - t0
    per_row = w.flops / (w.batch * w.Nq)           # mean over the rows (a causal row sees a part of the keys)
    rows = 64
    dt = run(rows)
    rows2 = int(min(w.batch * w.Nq, max(rows, rows * budget_s / max(dt, 1e-6))))
    if rows2 > 2 * rows:
        rows, dt = rows2, run(rows2)
    return {"value": rows * per_row / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{rows} query rows x {w.Nk} keys (D={w.D}), {dt:.1f} s", "seconds": dt}


def cpu_baseline(w, host, budget_s=15.0):
    """The oracle, as it stands, on a bounded slice of the same workload."""
    import numpy as np
    import oracle
    import workloads as wl
    if is_attention(w):
        return cpu_baseline_attention(w, host, budget_s)
    if is_int8(w):
        q = {k: host[k] for k in ("scale", "bias", "mid_scale", "mul", "add", "relu", "out_scale")}
        rows = 8
        t0 = time.perf_counter(); oracle.matmul_int8(host["a"][:rows], host["b"], trans_b=1, **q); dt = time.perf_counter() - t0
        rows2 = int(min(w.M, max(rows, rows * budget_s / max(dt, 1e-6))))
        if rows2 > 2 * rows:
            rows = rows2
            t0 = time.perf_counter(); oracle.matmul_int8(host["a"][:rows], host["b"], trans_b=1, **q); dt = time.perf_counter() - t0
        return {"value": 2.0 * rows * w.N * w.K / dt / 1e12, "unit": "TOP/s", "cores": oracle.num_threads(), "kind": "oracle",
                "sample": f"{rows} rows x {w.N} columns of the output (K={w.K}), {dt:.1f} s", "seconds": dt}
    threads = oracle.num_threads()
    m, n, k = w.gemm_mnk

    def run(rows, cols):
        t0 = time.perf_counter()
        if w.kind == "conv":
            # first `rows` output pixels of image 0 x all channels: use whole output rows
            nrow = max(1, rows // w.OW)
            Hs = min(w.H, (nrow - 1) * w.stride[0] + w.dil[0] * (w.KH - 1) + 1)
            xs = np.ascontiguousarray(host["a"][:1, :Hs])
            o = oracle.conv2d_nhwc(xs, host["b"], host["bias"], dtype=w.in_dtype, stride=w.stride,
                                   pad=(0, w.pad[1]), dil=w.dil, alpha=w.alpha, epi=w.epi)
            flops = 2.0 * o.shape[1] * o.shape[2] * n * k
            what = f"{o.shape[1]}x{o.shape[2]} output pixels of one image x {n} channels"
        else:
            a = host["a"].reshape(-1, k)[:rows]
            b = host["b"].reshape(-1, host["b"].shape[-1])[: (cols if w.trans_b else k)]
            oracle.matmul(a, b, host["bias"], dtype=w.in_dtype, trans_b=w.trans_b, alpha=w.alpha,
                          epi=w.epi, M=rows, N=cols, K=k, lda=k, ldb=host["b"].shape[-1])
            flops = 2.0 * rows * cols * k
            what = f"{rows} rows x {cols} columns of the output (K={k})"
        return time.perf_counter() - t0, flops, what

    rows, cols = min(m, 8), min(n, 512)
    dt, flops, what = run(rows, cols)
    rate = flops / max(dt, 1e-9)
    # grow the sample towards the time budget
    scale = budget_s * rate / flops
    if scale > 2:
        cols2 = int(min(n, cols * max(1.0, scale)))
        rows2 = int(min(m, max(rows, rows * scale * cols / cols2)))
        if w.kind == "conv":
            rows2 = int(min(w.OH * w.OW, rows2))
        dt, flops, what = run(rows2, cols2)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "sample": f"{what}, {dt:.1f} s", "seconds": dt}


def load_traffic(name):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if any."""
    p = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(p):
        with open(p) as f:
            return json.load(f).get(name)
    return None


def _pmc_child(counter, extra, outdir, tag, timeout_s):
    """One rocprofv3 --pmc run of this script as a child process; returns {kernel name: mean counter value}."""
    import csv
    import glob
    import shutil
    import subprocess
    exe = shutil.which("rocprofv3")
    if not exe:
        return None
    env = dict(os.environ, TMPDIR="/tmp")
    cmd = [exe, "--pmc", counter, "-d", outdir, "-o", tag, "--output-format", "csv", "--",
           sys.executable, os.path.abspath(__file__), *extra]
    try:
        subprocess.run(cmd, cwd="/tmp", env=env, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL,
                       timeout=timeout_s, check=True)
    except Exception:
        return None
    vals = {}
    for f in glob.glob(os.path.join(outdir, "**", tag + "_counter_collection.csv"), recursive=True):
        with open(f) as fh:
            for r in csv.DictReader(fh):
                if r["Counter_Name"] == counter:
                    vals.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in vals.items()} or None


def measure_traffic(workload, timeout_s=150):
    """HBM-side bytes per launch of the workload's kernel, measured now: FETCH_SIZE and WRITE_SIZE (KiB per
    dispatch) from one rocprofv3 --pmc child run each, scaled by what the same counters read for a 1 GiB
    device copy.  Must run before this process initialises the GPU.  None if the profiler is not usable."""
    import tempfile
    out = tempfile.mkdtemp(prefix="pbk_traffic_")
    res = {}
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        k = _pmc_child(counter, ["--workload", workload, "--steps", "3", "--warmup", "1", "--no-cpu-baseline",
                                 "--no-traffic", "--no-copy"], out, "w_" + counter, timeout_s)
        c = _pmc_child(counter, ["--calibrate-copy", "--steps", "2"], out, "c_" + counter, timeout_s)
        if not k or not c:
            return None
        ker = [v for n, v in k.items() if "pbk" in n]
        cop = [v for n, v in c.items() if "copy" in n.lower()]
        if not ker or not cop or cop[0] <= 0:
            return None
        scale = (1 << 20) / cop[0]                    # the copy moves 2^20 KiB each way
        res[counter] = max(ker) * 1024.0 * scale
        res[counter + "_scale"] = scale
    return {"bytes": res["FETCH_SIZE"] + res["WRITE_SIZE"], "fetch_bytes": res["FETCH_SIZE"],
            "write_bytes": res["WRITE_SIZE"], "fetch_scale": res["FETCH_SIZE_scale"],
            "write_scale": res["WRITE_SIZE_scale"]}


def report(w, r, steps, warmup, with_cpu=True, traffic=None, copy_bw=None):
    bound, peak = bound_of(w)
    avg_ms = sum(r["event_ms"]) / len(r["event_ms"])
    if bound == "mfma":
        achieved = w.flops / (avg_ms * 1e-3) / 1e12
        unit = "TFLOP/s"
    else:
        achieved = w.algorithmic_bytes / (avg_ms * 1e-3) / 1e9
        unit = "GB/s"
    line = {
        "metric": "TFLOP/s, fused matmul 8192^3 bf16 (1 GPU)" if w.name == HEADLINE
                  else f"TFLOP/s, {w.name} (1 GPU)",
        "value": w.flops / (r["wall_ms_per_step"] * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": r["wall_ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE_NAMES[in_dtype_of(w)], "data": "zeros (power-limit probe, not a benchmark result)" if ZERO_OPERANDS else "synthetic",
        "config": ({"workload": w.name, "kind": "matmul_int8", "gemm_mnk": [w.M, w.N, w.K], "trans_b": 1,
                    "epilogue": "dequant+bias+requant pair+affine+relu+quantise", "out_dtype": "int8",
                    "kernel": r["kernel"]} if is_int8(w) else
                   {"workload": w.name, "kind": "attention", "batch_x_heads": w.batch, "Nq": w.Nq, "Nk": w.Nk,
                    "D": w.D, "bias": w.bias, "causal": bool(w.causal), "kernel": r["kernel"]} if is_attention(w) else
                   {"workload": w.name, "kind": w.kind, "gemm_mnk": list(w.gemm_mnk), "batch": w.batch,
                    "epilogue": w.epi, "out_dtype": DTYPE_NAMES[w.out_dtype], "kernel": r["kernel"]}),
        "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                     "frac": achieved / peak,
                     "traffic": traffic["bytes"] if traffic else load_traffic(w.name),
                     "traffic_source": ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE child runs of this command, scaled by a "
                                        "1 GiB device copy" if traffic else "profiles/hbm_traffic.json (committed summary)"),
                     "kernel_ms_avg": avg_ms, "kernel_ms_min": min(r["event_ms"]),
                     "algorithmic_bytes": w.algorithmic_bytes, "flops": w.flops,
                     "buffer_sets": r.get("buffer_sets", 1)},
    }
    if traffic:
        line["roofline"]["traffic_detail"] = {k: traffic[k] for k in ("fetch_bytes", "write_bytes", "fetch_scale", "write_scale")}
    if bound == "hbm":
        line["roofline"]["mfma_frac"] = w.flops / (avg_ms * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS
    if copy_bw:
        # what a plain device copy / fill reaches in this run, beside the 8 TB/s of the data sheet
        line["roofline"]["copy_GBps"] = copy_bw["copy"]
        line["roofline"]["fill_GBps"] = copy_bw["fill"]
        if bound == "hbm":
            line["roofline"]["frac_of_copy"] = achieved / copy_bw["copy"]
    if with_cpu:
        line["cpu_baseline"] = cpu_baseline(w, r["host"])
    return line


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--all", action="store_true", help="also time the other workloads (table on stderr)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--json-out", default=None, help="with --all: also write every workload's line to this file")
    ap.add_argument("--table-out", default=None, help="with --all: also write the per-workload table to this text file")
    ap.add_argument("--extra", action="store_true", help="with --all: include the FP8, int8 and attention workloads")
    ap.add_argument("--no-traffic", action="store_true", help="do not measure HBM traffic with rocprofv3 child runs")
    ap.add_argument("--no-copy", action="store_true", help="do not time the device copy / fill")
    ap.add_argument("--zero-operands", action="store_true",
                    help="power-limit probe: time the same launches on all-zero operands (not a benchmark result: "
                         "the line is marked \"data\": \"zeros\")")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a 1 GiB device-to-device copy (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    global ZERO_OPERANDS
    ZERO_OPERANDS = args.zero_operands
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the contraction shards by output tiles without "
                 "any exchange; nothing multi-GPU is implemented). Use --gpus 1.")

    # HBM traffic counters: child runs under the profiler, before this process touches the GPU
    traffic = None
    if not (args.no_traffic or args.calibrate_copy or args.all or args.zero_operands):
        traffic = measure_traffic(args.workload)

    import torch
    import workloads as wl
    import paper_2603_06731_amd as pbk
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    pbk.lib()       # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "launches": args.steps}))
        return

    w = {**wl.CONFIGS, **wl.EXTRA_CONFIGS, **wl.ATTENTION_CONFIGS, **wl.INT8_CONFIGS}[args.workload]
    copy_bw = None if args.no_copy else measure_copy_bandwidth()
    r = time_workload(w, args.steps, args.warmup)
    line = report(w, r, args.steps, args.warmup, with_cpu=not args.no_cpu_baseline, traffic=traffic, copy_bw=copy_bw)
    del r

    if args.all:
        rows = [line]
        pool = dict(wl.CONFIGS)
        if args.extra:
            pool.update({**wl.EXTRA_CONFIGS, **wl.INT8_CONFIGS,
                         **{k: v for k, v in wl.ATTENTION_CONFIGS.items() if "8192" in k or "2048" in k}})
        for name, ww in pool.items():
            if name == args.workload:
                continue
            rr = time_workload(ww, args.steps, args.warmup)
            rows.append(report(ww, rr, args.steps, args.warmup, with_cpu=not args.no_cpu_baseline, copy_bw=copy_bw))
            del rr
        table = []
        for x in rows:
            rf = x["roofline"]
            extra = f"  ({rf['frac_of_copy']*100:.1f}% of this run's device copy)" if "frac_of_copy" in rf else ""
            table.append(f"{x['config']['workload']:24s} {x['config']['kernel']:36s} {rf['kernel_ms_avg']*1e3:9.1f} us (min "
                         f"{rf['kernel_ms_min']*1e3:7.1f})  {x['value']:8.1f} TFLOP/s  {rf['bound']}: {rf['achieved']:.1f} "
                         f"{rf['unit']} = {rf['frac']*100:.1f}% of {rf['peak']:g}  sets={rf['buffer_sets']}{extra}")
        print("\n".join(table), file=sys.stderr)
        if args.table_out:
            with open(args.table_out, "w") as f:
                f.write("python bench.py " + " ".join(sys.argv[1:]) + "\n")
                f.write("kernel time: HIP events around every launch, mean (min) over the timed steps; TFLOP/s from wall time\n")
                if copy_bw:
                    f.write(f"device copy of 1 GiB in this run: {copy_bw['copy']:.0f} GB/s (read + write), fill {copy_bw['fill']:.0f} GB/s\n")
                f.write("\n".join(table) + "\n")
        if args.json_out:
            with open(args.json_out, "w") as f:
                json.dump(rows, f, indent=1)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
