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
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        st, _o = run(w, dev, out=out, stream=stream)
        pbk.check(st, w.name)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        starts[i].record(stream)
        st, _o = run(w, dev, out=out, stream=stream)
        ends[i].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    pbk.check(st, w.name)
    ev_ms = [s.elapsed_time(e) for s, e in zip(starts, ends)]
    return {"wall_ms_per_step": (t1 - t0) * 1e3 / steps, "event_ms": ev_ms,
            "kernel": pbk.pbk_last_kernel(), "host": host, "out": out}


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
        oracle.attention_rows(host["q"], host["k"], host["v"], host["bias"], sb, si, dtype=w.dtype, alpha=w.alpha)
        return time.perf_counter() - t0
    per_row = 4.0 * w.Nk * w.D
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


def report(w, r, steps, warmup, with_cpu=True):
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
        "dtype": DTYPE_NAMES[in_dtype_of(w)], "data": "synthetic",
        "config": ({"workload": w.name, "kind": "matmul_int8", "gemm_mnk": [w.M, w.N, w.K], "trans_b": 1,
                    "epilogue": "dequant+bias+requant pair+affine+relu+quantise", "out_dtype": "int8",
                    "kernel": r["kernel"]} if is_int8(w) else
                   {"workload": w.name, "kind": "attention", "batch_x_heads": w.batch, "Nq": w.Nq, "Nk": w.Nk,
                    "D": w.D, "bias": w.bias, "kernel": r["kernel"]} if is_attention(w) else
                   {"workload": w.name, "kind": w.kind, "gemm_mnk": list(w.gemm_mnk), "batch": w.batch,
                    "epilogue": w.epi, "out_dtype": DTYPE_NAMES[w.out_dtype], "kernel": r["kernel"]}),
        "roofline": {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit,
                     "frac": achieved / peak, "traffic": load_traffic(w.name),
                     "kernel_ms_avg": avg_ms, "kernel_ms_min": min(r["event_ms"]),
                     "algorithmic_bytes": w.algorithmic_bytes, "flops": w.flops},
    }
    if bound == "hbm":
        line["roofline"]["mfma_frac"] = w.flops / (avg_ms * 1e-3) / 1e12 / PEAK_MFMA_16BIT_TFLOPS
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
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a 1 GiB device-to-device copy (reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (the contraction shards by output tiles without "
                 "any exchange; nothing multi-GPU is implemented). Use --gpus 1.")

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
    r = time_workload(w, args.steps, args.warmup)
    line = report(w, r, args.steps, args.warmup, with_cpu=not args.no_cpu_baseline)
    del r

    if args.all:
        rows = [line]
        for name, ww in wl.CONFIGS.items():
            if name == args.workload:
                continue
            rr = time_workload(ww, args.steps, args.warmup)
            rows.append(report(ww, rr, args.steps, args.warmup, with_cpu=not args.no_cpu_baseline))
            del rr
        for x in rows:
            rf = x["roofline"]
            print(f"{x['config']['workload']:24s} {x['config']['kernel']:26s} {rf['kernel_ms_avg']*1e3:9.1f} us  "
                  f"{x['value']:8.1f} TFLOP/s  {rf['bound']}: {rf['achieved']:.1f} {rf['unit']} = {rf['frac']*100:.1f}%",
                  file=sys.stderr)
        if args.json_out:
            with open(args.json_out, "w") as f:
                json.dump(rows, f, indent=1)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
