#!/usr/bin/env python3
"""Benchmarks of the LQ decomposition path on one MI355X.  Every mode prints one JSON line.

--workload sweep (default): one step = the whole hot path over one of the five benchmark workloads (--config):
  1  one 768 x 768 matrix, rank 8, NF3 B0 = 64 B1 = 256, 5 LQ iterations (one lq_decompose call)
  2  RoBERTa-Large-shaped stack, 24 blocks x (4x 1024x1024, 1024x4096, 4096x1024), rank 8, 9 configurations
     (bits 2/3/4 x B0 16/32/64, B1 = 256), 10 iterations: one lq_error_table call per matrix
  3  (default, the headline metric) one LLaMA-2-7B-shaped block (4x 4096x4096, 2x 4096x11008, 11008x4096), rank 64,
     36 configurations (bits 2/3/4/8 x B0 16/32/64 x B1 16/64/256), 10 iterations
  4  one Fisher-weighted 4096 x 11008 matrix, rank 64, NF3 64/256, 10 iterations (one weighted lq_decompose call)
  5  one LLaMA-2-70B-shaped block (2x 8192x8192, 2x 8192x1024, 2x 8192x28672, 28672x8192), rank 64, 36 configurations
--workload quant: the other half of the metric, lq_nf_quantize / lq_nf_dequantize in algorithmic GB/s over the
  matrix shapes of workloads 3 and 5, buffers rotated so that nothing stays in the 256 MB Infinity Cache.
--workload matmul: the consumer of a decomposition, Y = X (Q + L1 L2) with just-in-time dequantization.
Inputs are synthetic (paper_2311_12023_amd/gen.py) and resident in HBM before the timed region.
"""
from __future__ import annotations

import argparse
import json
import os
import queue
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_HBM_GBS = 8000.0

ROBERTA_GRID = [(b, b0, 256) for b in (2, 3, 4) for b0 in (16, 32, 64)]
NF3_DEFAULT = (3, 64, 256)

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "llama7b_layer_sweep_hbm_traffic.md")
FORWARD_TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "llama7b_layer_forward_kernel_stats.md")
QUANT_TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "nf_quantize_dequantize_kernel_stats.md")


def host_cores() -> int:
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    return min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))


def measured_traffic(name: str, table: str | None = None):
    """HBM-side bytes per launch of a kernel class (fetch + write) from a committed counter summary, averaged over
    the class's template variants weighted by launches; None when the summary does not list the kernel."""
    try:
        lines = open(table or TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None
    base = name.split("<")[0]
    want = name.replace(" ", "")
    tot = n = 0.0
    parts = 0.0          # residual_kernel: one launch of the class is one launch per code width; their traffic adds up
    # a summary that also holds other tables marks the counter table with a heading that names the traffic
    headed = any(ln.startswith("#") and "traffic" in ln.lower() for ln in lines[1:])
    inside = not headed
    for ln in lines:
        if headed and ln.startswith("#"):
            inside = "traffic" in ln.lower()
        cells = [c.strip() for c in ln.strip().strip("|").split("|")]
        if not inside or len(cells) != 4 or not cells[0].startswith("`"):
            continue
        kern = cells[0].strip("`").replace(" ", "")
        per_launch = (float(cells[2]) + float(cells[3])) * 1e6
        if name.startswith("wide_gemm"):
            hit = kern.startswith(want[:-1] + ",")          # the table's names carry one more template argument
        elif base == "lowrank_blockquant_kernel":
            hit = kern.startswith("lowrank_blockquant")
        elif base == "residual_kernel":
            if kern.startswith("residual_planes_kernel"):
                parts += per_launch
            hit = kern.split("<")[0] == base
        else:
            hit = kern.split("<")[0] == base
        if hit:
            launches = float(cells[1])
            tot += launches * per_launch
            n += launches
    if parts:
        return parts
    return tot / n if n else None


# Kernel classes with a roofline of their own.  Everything else the library launches (Gram matrices, Cholesky, Jacobi,
# fix-ups, packing) is a short or single-workgroup kernel bound by latency; those are listed with their time only.
STREAMING = ("lowrank_blockquant_kernel", "residual_kernel", "scalequant_error_kernel", "quantize_fused_kernel",
             "dequant_kernel")


def roofline_of(name: str, ms: float, launches: int, work: float) -> dict | None:
    """Roofline entry of one kernel class from its summed HIP-event time and algorithmic work (what the operation
    has to move or multiply, not what the kernel happened to move)."""
    if ms <= 0 or launches <= 0:
        return None
    sec = ms * 1e-3
    common = {"kernel": name, "traffic": None, "launches": launches, "avg_us": 1e3 * ms / launches}
    if name.startswith("wide_gemm_f16_kernel"):
        # A as an fp16 plane (2 B per element) or as that plane plus a byte plane (3 B), 2 l flop per element; one plane: X
        # rounded to fp16, one MFMA per product; two planes: X split into fp16 hi + lo, three MFMAs per product; bound by
        # streaming A
        lt, _, planes = (int(t) for t in name[name.index("<") + 1:name.index(">")].split(","))
        ach = work / (2.0 * 32 * lt) * (2.0 if planes == 1 else 3.0) / sec / 1e9
        return {**common, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                "algorithmic_tflops": work / sec / 1e12,
                "executed_f16_mfma_frac": (1.0 if planes == 1 else 3.0) * work / sec / 1e12 / PEAK_BF16_MFMA_TFLOPS}
    if name.startswith("wide_gemm_kernel"):
        lt, _, _, prec = (int(t) for t in name[name.index("<") + 1:name.index(">")].split(","))
        if prec == 0:      # fp32 MFMA: work is flops
            ach = work / sec / 1e12
            return {**common, "bound": "mfma", "achieved": ach, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / PEAK_FP32_MFMA_TFLOPS}
        # split mode: every product is three bf16 MFMAs; the operand A (4 B per element, 2 l flop per element) is
        # streamed once, which is what bounds the kernel
        ach = work / (2.0 * 32 * lt) * 4.0 / sec / 1e9
        return {**common, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                "algorithmic_tflops": work / sec / 1e12,
                "executed_bf16_mfma_frac": 3.0 * work / sec / 1e12 / PEAK_BF16_MFMA_TFLOPS}
    if name.split("+")[0] in STREAMING:
        ach = work / sec / 1e9
        return {**common, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}
    return None


def dominant_roofline(prof: dict):
    """-> (roofline of the class with the largest summed time among those that have one, share of the summed kernel
    time spent in latency-bound classes)."""
    total = sum(v[0] for v in prof.values())
    best = None
    lat = 0.0
    for name, (ms, n, work) in prof.items():
        r = roofline_of(name, ms, n, work)
        if r is None:
            lat += ms
        elif best is None or ms > best[0]:
            best = (ms, r)
    return (best[1] if best else None), (lat / total if total > 0 else 0.0)


# ------------------------------------------------------------------------------------------------------------------
# CPU baselines: the oracle as it stands on a bounded sample
def cpu_baseline_lq(sample: np.ndarray, rank: int, cfg_tuple, iters: int, what: str, row_w=None, col_w=None) -> dict:
    from oracle import lq_oracle as O
    O.build()
    t0 = time.perf_counter()
    O.lq(sample, rank, O.config(*cfg_tuple), iters, row_w=row_w, col_w=col_w)
    dt = time.perf_counter() - t0
    return {"value": 1.0 / dt, "unit": "matrix-configs/s on the sample", "cores": host_cores(), "kind": "oracle",
            "sample": f"{what}: {dt:.1f} s"}


def cpu_baseline_quant(sample: np.ndarray, cfg_tuple) -> dict:
    from oracle import lq_oracle as O
    O.build()
    cfg = O.config(*cfg_tuple)
    flat = np.ascontiguousarray(sample.ravel())
    t0 = time.perf_counter()
    codes, sidx, v, _ = O.quantize(flat, cfg)
    t1 = time.perf_counter()
    O.dequantize(codes, sidx, v, cfg)
    t2 = time.perf_counter()
    b = quant_bytes(flat.size, cfg_tuple)
    return {"value": 2.0 * b / (t2 - t0) / 1e9, "unit": "GB/s", "cores": host_cores(), "kind": "oracle",
            "sample": f"quantize + dequantize of one {sample.shape[0]}x{sample.shape[1]} matrix, NF{cfg_tuple[0]} "
                      f"B0={cfg_tuple[1]} B1={cfg_tuple[2]} (brute-force nearest code): {t1 - t0:.2f} s + {t2 - t1:.2f} s"}


def quant_bytes(n: int, cfg_tuple) -> float:
    """Algorithmic bytes of one Quantize (or Dequantize) of n weights: fp32 on one side, codes, one byte per block scale
    and one fp32 per scale group on the other."""
    b0, blk, sblk = cfg_tuple[:3]
    return n * (4.0 + b0 / 8.0 + 1.0 / blk + 4.0 / (blk * sblk))


# ------------------------------------------------------------------------------------------------------------------
def bench_quant(args, torch, gen, lq, dev) -> int:
    """lq_nf_quantize and lq_nf_dequantize over the distinct matrix shapes of workloads 3 and 5 for the corners of the
    configuration grid.  One step = every (shape, configuration) cell quantized and dequantized once."""
    shapes = [(3, 0, "4096x4096"), (3, 4, "4096x11008"), (5, 0, "8192x8192"), (5, 4, "8192x28672")]
    if args.matrices < len(shapes):
        shapes = shapes[:args.matrices]
    grid = [(2, 16, 16), (2, 64, 256), NF3_DEFAULT, (4, 64, 256), (8, 16, 16), (8, 64, 256)]
    rotate_bytes = 1.5e9            # every buffer class cycles through at least this much memory
    cells = []
    host0 = None
    for wl, idx, label in shapes:
        w = gen.workload_matrix(wl, idx)
        if host0 is None:
            host0 = w
        n = w.size
        copies = max(2, int(np.ceil(rotate_bytes / (4.0 * n))))
        xs = [torch.from_numpy(w).to(dev).reshape(-1)]
        for _ in range(copies - 1):
            xs.append(xs[0].clone())
        outs = [torch.empty(n, dtype=torch.float32, device=dev) for _ in range(copies)]
        for g in grid:
            cfg = lq.config(*g)
            packs = [lq.nf_quantize(xs[0], cfg) for _ in range(copies)]
            cells.append(dict(label=label, n=n, g=g, cfg=cfg, xs=xs, outs=outs, packs=packs, copies=copies))
        del w
    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.mul(src, 2.0, out=dst)          # one elementwise kernel: 1 GiB in, 1 GiB out
        torch.cuda.synchronize()
        del src, dst
    counter = [0]

    def step():
        counter[0] += 1
        for c in cells:
            i = counter[0] % c["copies"]
            lq.nf_quantize(c["xs"][i], c["cfg"], out=c["packs"][i])
        for c in cells:
            i = counter[0] % c["copies"]
            lq.nf_dequantize(*c["packs"][i], c["n"], c["cfg"], out=c["outs"][i])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec = time.perf_counter() - t0
    total_bytes = 2.0 * sum(quant_bytes(c["n"], c["g"]) for c in cells)
    # per-cell durations: for each cell a run of back-to-back calls over the rotated buffers between two events (a single
    # call of 15 - 250 us bracketed on an otherwise idle GPU would mostly measure launch latency and the clock ramp)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    per_cell = []
    for c in cells:
        reps = max(4, 2 * c["copies"])
        times = []
        for which in (0, 1):
            for timed in (False, True):
                a, b = ev(), ev()
                a.record()
                for r in range(reps):
                    i = r % c["copies"]
                    if which == 0:
                        lq.nf_quantize(c["xs"][i], c["cfg"], out=c["packs"][i])
                    else:
                        lq.nf_dequantize(*c["packs"][i], c["n"], c["cfg"], out=c["outs"][i])
                b.record()
                torch.cuda.synchronize()
                if timed:
                    times.append(a.elapsed_time(b) / reps)
        tq, td = times
        by = quant_bytes(c["n"], c["g"])
        per_cell.append({"shape": c["label"], "config": list(c["g"]), "bytes": by,
                         "quantize_us": 1e3 * tq, "dequantize_us": 1e3 * td,
                         "quantize_GBs": by / (tq * 1e-3) / 1e9, "dequantize_GBs": by / (td * 1e-3) / 1e9})
    lq.profile_enable(True)
    lq.profile_reset()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = lq.profile_read()
    lq.profile_enable(False)
    roofs = {n: roofline_of(n, *v) for n, v in prof.items()}
    roofs = {n: r for n, r in roofs.items() if r}
    dom = max(roofs.values(), key=lambda r: r["avg_us"] * r["launches"]) if roofs else None
    if dom is not None and len(shapes) == 4:
        dom["traffic"] = measured_traffic(dom["kernel"], QUANT_TRAFFIC_TABLE)
    big = [p for p in per_cell if p["shape"] != "4096x4096"]
    out = {"metric": "NF quant HBM GB/s (lq_nf_quantize + lq_nf_dequantize, algorithmic bytes)",
           "value": total_bytes * args.steps / sec / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": 1e3 * sec / args.steps, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "Quantize and Dequantize (Section 3.2) of " + ", ".join(s[2] for s in shapes)
                                  + " matrices (workload 3 and 5 shapes) for " + ", ".join(f"NF{g[0]} {g[1]}/{g[2]}" for g in grid),
                      "cells": len(cells), "rotation": "each buffer class cycles through >= 1.5 GB"},
           "roofline": dom,
           "roofline_note": "algorithmic bytes per call = n (4 + b0/8 + 1/B0 + 4/(B0 B1)); roofline = the kernel class "
                            "with the larger summed time, durations from a pass of the same steps with every launch "
                            "bracketed by events on its stream; value from the pass without brackets",
           "roofline_kernels": roofs,
           "quantize_frac_of_hbm_min_max": [min(p["quantize_GBs"] for p in big) / PEAK_HBM_GBS,
                                            max(p["quantize_GBs"] for p in big) / PEAK_HBM_GBS] if big else None,
           "dequantize_frac_of_hbm_min_max": [min(p["dequantize_GBs"] for p in big) / PEAK_HBM_GBS,
                                              max(p["dequantize_GBs"] for p in big) / PEAK_HBM_GBS] if big else None,
           "cells": per_cell}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_quant(host0, NF3_DEFAULT)
    print(json.dumps(out))
    return 0


# ------------------------------------------------------------------------------------------------------------------
NF4_DOUBLE_QUANT = (4, 64, 256, 8, "bf16")


def bench_matmul(args, torch, gen, lq, dev) -> int:
    """Forward products Y = X (Q + L1 L2) of one LLaMA-2-7B-shaped layer; one step = all 7 matrices."""
    RANK = 64
    shapes = gen.LLAMA2_7B_LAYER[:args.matrices]
    cfg = lq.config(*NF4_DOUBLE_QUANT)
    m = args.tokens
    acts = {d: torch.from_numpy(gen.activations(m, d, gen.matrix_seed(3, 900 + i))).to(dev)
            for i, d in enumerate(sorted({d for d, _ in shapes}))}
    items = []
    for i, (d, k) in enumerate(shapes):
        w = torch.from_numpy(gen.workload_matrix(3, i)).to(dev)
        codes, sidx, v = lq.nf_quantize(w.reshape(-1), cfg)
        l1, l2 = (torch.from_numpy(a).to(dev) for a in gen.low_rank_factors(d, k, RANK, gen.matrix_seed(3, 800 + i)))
        items.append(dict(d=d, k=k, codes=codes, sidx=sidx, v=v, l1=l1, l2=l2, x=acts[d],
                          out=torch.empty((m, k), dtype=torch.float32, device=dev),
                          ws=lq.matmul_workspace(m, d, k, RANK, dev)))
        del w
    flops = sum(2.0 * m * it["d"] * it["k"] + 2.0 * m * RANK * (it["d"] + it["k"]) for it in items)

    def step():
        for it in items:
            lq.matmul(it["x"], it["codes"], it["sidx"], it["v"], cfg, it["k"], it["l1"], it["l2"],
                      precision=args.precision, out=it["out"], workspace=it["ws"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    sec = time.perf_counter() - t0
    # kernel durations: the same steps once more with every launch bracketed by two events on its stream (the brackets
    # cost several microseconds per launch, which would distort the timed region of a workload of short kernels)
    prof = {}
    if not args.no_profile:
        lq.profile_enable(True)
        lq.profile_reset()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        prof = lq.profile_read()
        lq.profile_enable(False)
    ms = 1e3 * sec / args.steps
    out = {"metric": "fp32-grade TFLOP/s of the forward product X (Q + L1 L2) with just-in-time dequantization",
           "value": flops / (sec / args.steps) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16x3" if args.precision == 0 else "bf16", "data": "synthetic",
           "config": {"workload": f"LLaMA-2-7B layer forward, {m} tokens, {len(items)} matrices, NF4 + double "
                                  f"quantization, rank {RANK}"}}
    if "qmatmul_kernel" in prof:
        kms, launches, work = prof["qmatmul_kernel"]
        mult = 3.0 if args.precision == 0 else 1.0          # bf16 MFMAs executed per product
        ach = mult * work / (kms * 1e-3) / 1e12
        traffic = None
        if m == 4096 and len(items) == 7 and args.precision == 0:      # the configuration the counter runs measured
            traffic = measured_traffic("qmatmul_kernel", FORWARD_TRAFFIC_TABLE)
        out["roofline"] = {"kernel": "qmatmul_kernel", "bound": "mfma", "achieved": ach, "peak": PEAK_BF16_MFMA_TFLOPS,
                           "unit": "TFLOP/s", "frac": ach / PEAK_BF16_MFMA_TFLOPS, "traffic": traffic,
                           "launches": launches, "avg_us": 1e3 * kms / launches,
                           "algorithmic_tflops": work / (kms * 1e-3) / 1e12}
        out["roofline_note"] = ("achieved counts the bf16 MFMA flops the kernel executes (3 per product at precision 0) "
                                "against the dense bf16 peak; algorithmic_tflops counts each product once.  Kernel "
                                "durations come from a second pass over the same steps with every launch bracketed by "
                                "events on the launch stream; value and ms_per_step from the pass without brackets.")
        out["kernels"] = {n: {"ms": v[0], "launches": v[1]} for n, v in prof.items()}
    elif "qmatvec_kernel" in prof:                           # few tokens: bound by reading the weights once
        kms, launches, work = prof["qmatvec_kernel"]
        ach = work / (kms * 1e-3) / 1e9
        out["dtype"] = "f32"
        out["roofline"] = {"kernel": "qmatvec_kernel", "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS,
                           "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "traffic": None, "launches": launches,
                           "avg_us": 1e3 * kms / launches}
        out["roofline_note"] = ("algorithmic bytes per launch: the packed codes and one scale index per block of the "
                                "d x k matrix, both low-rank factors, X and Y.  Kernel durations come from a second pass "
                                "over the same steps with every launch bracketed by events (an upper bound for kernels "
                                "this short); value and ms_per_step from the pass without brackets.")
        out["kernels"] = {n: {"ms": v[0], "launches": v[1]} for n, v in prof.items()}
    if not args.no_cpu_baseline:
        from oracle import lq_oracle as O
        it = items[0]
        rows = min(4, m)
        codes = O.unpack(it["codes"].cpu().numpy(), it["d"] * it["k"], 4)
        t0 = time.perf_counter()
        O.matmul(it["x"][:rows].cpu().numpy(), codes, it["sidx"].cpu().numpy(), it["v"].cpu().numpy(),
                 O.config(*NF4_DOUBLE_QUANT), it["k"], it["l1"].cpu().numpy(), it["l2"].cpu().numpy())
        cs = time.perf_counter() - t0
        cfl = 2.0 * it["d"] * it["k"] * (rows + RANK)        # forming Q + L1 L2 and the product of `rows` rows
        out["cpu_baseline"] = {"value": cfl / cs / 1e12, "unit": "TFLOP/s", "cores": 1, "kind": "oracle",
                               "sample": f"{rows} rows of X against the first {it['d']}x{it['k']} matrix "
                                         f"(fp64 definition, Q + L1 L2 formed densely): {cs:.1f} s"}
    print(json.dumps(out))
    return 0


# ------------------------------------------------------------------------------------------------------------------
class Workers:
    """Host threads that live for the whole benchmark, each with its own stream and workspace; run(jobs) hands the
    jobs out largest first and returns when all are done."""

    def __init__(self, torch, dev, workspaces):
        self.torch = torch
        self.n = len(workspaces)
        self.workspaces = workspaces
        self.streams = [torch.cuda.Stream(device=dev) for _ in workspaces]
        self.todo: queue.Queue = queue.Queue()
        self.done: queue.Queue = queue.Queue()
        self.threads = [threading.Thread(target=self._loop, args=(t,), daemon=True) for t in range(self.n)]
        for th in self.threads:
            th.start()

    def _loop(self, tid):
        with self.torch.cuda.stream(self.streams[tid]):
            while True:
                job = self.todo.get()
                if job is None:
                    return
                key, fn, limit = job
                if tid >= limit:                 # this pass runs on fewer threads: leave the job to them
                    self.todo.put(job)
                    time.sleep(0.001)
                    continue
                try:
                    self.done.put((key, fn(self.workspaces[tid]), None))
                except Exception as exc:     # surfaced by run()
                    self.done.put((key, None, exc))

    def run(self, jobs, threads=None):
        limit = self.n if threads is None else max(1, min(threads, self.n))
        for key, fn in jobs:
            self.todo.put((key, fn, limit))
        out = {}
        for _ in jobs:
            key, res, exc = self.done.get()
            if exc is not None:
                raise exc
            out[key] = res
        return out

    def close(self):
        for _ in self.threads:
            self.todo.put(None)
        for th in self.threads:
            th.join()


def bench_sweep(args, torch, gen, lq, dev) -> int:
    wl = args.config
    serial_params = lq.SvdParams(streams=1, gemm_mode=args.gemm_mode, first_width=args.first_width)
    params = lq.SvdParams(streams=args.streams, gemm_mode=args.gemm_mode, first_width=args.first_width)
    if wl in (1, 4):
        # one matrix, one configuration: a single lq_decompose call per step
        rank, iters = (8, 5) if wl == 1 else (64, 10)
        host = gen.workload_matrix(wl, 0)
        w = torch.from_numpy(host).to(dev)
        rw = cw = None
        if wl == 4:
            f = torch.from_numpy(gen.fisher_matrix(*host.shape, gen.matrix_seed(4, 1)).astype(np.float32)).to(dev)
            rw, cw = lq.fisher_row_col(f)       # set-up, not timed (Section 3.3: F comes from calibration gradients)
            del f
        cfg = lq.config(*NF3_DEFAULT)
        ws = torch.empty(lq._lib.lq_decompose_workspace_bytes(host.shape[0], host.shape[1], rank, None) + 256,
                         dtype=torch.uint8, device=dev)
        res = [None]

        def step(profiled_serial=False):
            res[0] = lq.decompose(w, rank, cfg, iters, row_w=rw, col_w=cw, seed=1, workspace=ws,
                                  params=serial_params if profiled_serial else None)
        cells, n_mats, n_cfgs, nthreads = 1, 1, 1, 1
        label = ("one 768x768 matrix, rank 8, NF3 B0=64 B1=256, 5 LQ iterations" if wl == 1 else
                 "one Fisher-weighted 4096x11008 matrix, rank 64, NF3 B0=64 B1=256, 10 LQ iterations (weighted error)")
        checksum = lambda: float(res[0]["err"])
        workers = None
    else:
        rank, iters = (8, 10) if wl == 2 else (64, 10)
        if wl == 2:
            count, grid = 24 * len(gen.ROBERTA_LARGE_LAYER), ROBERTA_GRID
        elif wl == 3:
            count, grid = len(gen.LLAMA2_7B_LAYER), (gen.paper_config_grid() if args.grid == "paper243" else gen.config_grid())
        else:
            count, grid = len(gen.LLAMA2_70B_LAYER), gen.config_grid()
        count = min(count, args.matrices)
        cfgs = [lq.config(*g) for g in grid]
        host0 = gen.workload_matrix(wl, 0)
        mats = [torch.from_numpy(host0 if i == 0 else gen.workload_matrix(wl, i)).to(dev) for i in range(count)]
        host = host0
        shapes = {tuple(m.shape) for m in mats}
        default_overlap = {2: 7, 3: 7, 5: 2}[wl]
        nthreads = max(1, min(args.overlap or default_overlap, len(mats)))
        # one workspace per concurrent matrix, each large enough for every shape of the workload
        need = max(lq._lib.lq_error_table_workspace_bytes(d, k, rank, len(cfgs), lq._pp(params)) for d, k in shapes)
        workers = Workers(torch, dev, [torch.empty(need + 256, dtype=torch.uint8, device=dev) for _ in range(nthreads)])
        order = sorted(range(len(mats)), key=lambda i: -mats[i].numel())      # largest first
        res = [None]

        def step(profiled_serial=False):
            p = serial_params if profiled_serial else params
            jobs = [(i, (lambda ws, i=i: lq.error_table(mats[i], rank, cfgs, iters, seed=1, params=p, workspace=ws)))
                    for i in order]
            res[0] = workers.run(jobs, threads=1 if profiled_serial else None)
        n_mats, n_cfgs = len(mats), len(cfgs)
        cells = n_mats * n_cfgs
        shape_text = {2: "RoBERTa-Large-shaped stack (24 blocks x (4x1024x1024, 1024x4096, 4096x1024)), rank 8, 9 configs "
                         "(bits 2/3/4 x B0 16/32/64, B1 256)",
                      3: "LLaMA-2-7B-shaped layer (4x4096x4096, 2x4096x11008, 1x11008x4096), rank 64, "
                         + ("36 configs (bits 2/3/4/8 x B0 16/32/64 x B1 16/64/256)" if args.grid == "sweep36" else
                            "243 configs (b0, b1 in 2/3/4 x b2 in bf16/fp16/fp32 x B0 16/32/64 x B1 16/64/256)"),
                      5: "LLaMA-2-70B-shaped layer (2x8192x8192, 2x8192x1024, 2x8192x28672, 1x28672x8192), rank 64, "
                         "36 configs (bits 2/3/4/8 x B0 16/32/64 x B1 16/64/256)"}[wl]
        label = shape_text + ", 10 LQ iterations"
        checksum = lambda: float(sum(np.sqrt(res[0][i][0]).sum() for i in range(len(mats))))

    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.mul(src, 2.0, out=dst)          # one elementwise kernel: 1 GiB in, 1 GiB out
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    check = checksum()
    # Kernel durations come from one more step with every launch bracketed by events on its stream, run one matrix at a
    # time on one stream so that every kernel has the GPU to itself (in the timed region up to four kernels of different
    # matrices share the compute units, and a bracket there measures the sharing, not the kernel).
    prof = {}
    if not args.no_profile:
        lq.profile_enable(True)
        lq.profile_reset()
        t1 = time.perf_counter()
        step(profiled_serial=True)
        torch.cuda.synchronize()
        serial_ms = 1e3 * (time.perf_counter() - t1)
        prof = lq.profile_read()
        lq.profile_enable(False)
    if workers is not None:
        workers.close()
    lq.release_streams()

    roof, latency_share = dominant_roofline(prof) if prof else (None, None)
    if roof is not None and wl == 3 and n_mats == 7 and args.grid == "sweep36":
        # the counter runs were taken in the default launch configuration (18 configurations per launch); the launches
        # timed here serve 36, and every byte of these kernels scales with the configurations served
        tr = measured_traffic(roof["kernel"])
        roof["traffic"] = None if tr is None else 2.0 * tr
        roof["traffic_note"] = ("FETCH_SIZE + WRITE_SIZE per launch of 18 configurations from "
                                "profiles/llama7b_layer_sweep_hbm_traffic.md, times two for the 36 served per launch here")
    split = args.gemm_mode != 1
    line = {
        "metric": "matrix-configs decomposed/sec" + (" (LLaMA-2-7B layer sweep)" if wl == 3 else f" (workload {wl})"),
        "value": cells * args.steps / dt, "unit": "matrix-configs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("f32 (large products: three bf16 MFMAs on hi/lo splits against fp32 operands; against the residual kept "
                  "as an fp16 plane plus a byte plane of what its rounding dropped, one fp16 MFMA on the fp16 plane where the "
                  "product only steers the subspace, three on both planes for the projection the results are read from; fp32 "
                  "accumulation)") if split else "f32",
        "data": "synthetic",
        "config": {"workload": label, "baseline_config": wl, "matrices": n_mats, "configs": n_cfgs, "iters": iters,
                   "rank": rank, "concurrent_matrices": nthreads,
                   "hip_hardware_queues": args.hw_queues},
        "roofline": roof,
        "roofline_note": "the kernel class with the largest summed duration among the machine-filling classes (large "
                         "GEMMs against HBM for the operand they stream, with the executed 16-bit MFMA work beside it; the "
                         "quantize / residual classes against HBM with their algorithmic bytes).  Durations are from "
                         "one extra step run one matrix at a time on one stream with every launch bracketed by events "
                         "(the kernel has the GPU to itself, as in the committed rocprofv3 table of that mode); value "
                         "and ms_per_step are from the steps without brackets.",
        "error_checksum": check,
    }
    if prof:
        line["serial_profiled_step_ms"] = serial_ms
        line["latency_bound_kernel_share"] = latency_share
        line["roofline_kernels"] = {n: r for n, r in ((n, roofline_of(n, *v)) for n, v in prof.items() if v[0] > 0.5) if r}
        line["kernels"] = {n: {"ms": round(v[0], 3), "launches": v[1]} for n, v in prof.items()}
    if not args.no_cpu_baseline:
        if wl == 1:
            line["cpu_baseline"] = cpu_baseline_lq(host, 8, NF3_DEFAULT, 5, "the whole workload (768x768, rank 8, NF3 64/256, "
                                                   "5 iterations, exact Jacobi SVD each)")
        elif wl == 2:
            line["cpu_baseline"] = cpu_baseline_lq(host, 8, NF3_DEFAULT, 10, "one cell of the table: matrix 0 (1024x1024), rank 8, "
                                                   "NF3 B0=64 B1=256, 10 iterations (exact Jacobi SVD each); the workload has 1296 "
                                                   "cells, a third of them on four times larger matrices")
        elif wl == 4:
            s = np.ascontiguousarray(host[:768, :1024])
            line["cpu_baseline"] = cpu_baseline_lq(s, 64, NF3_DEFAULT, 10, "the 768x1024 corner of the matrix, rank 64, NF3 64/256, "
                                                   "10 weighted iterations (exact Jacobi SVD each); the full matrix is 57 times "
                                                   "larger and its SVD cost grows with the 1.5th power of that",
                                                   row_w=rw.cpu().numpy()[:768], col_w=cw.cpu().numpy()[:1024])
        else:
            s = np.ascontiguousarray(host[:1024, :1024])
            line["cpu_baseline"] = cpu_baseline_lq(s, 64, NF3_DEFAULT, 10, "one 1024x1024 corner of matrix 0, rank 64, NF3 B0=64 "
                                                   "B1=256, 10 iterations (exact Jacobi SVD each); a full 4096x4096 cell costs "
                                                   "about 4^3 = 64 times as much")
    print(json.dumps(line))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default depends on the workload)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps first")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--config", type=int, choices=(1, 2, 3, 4, 5), default=3,
                    help="benchmark workload of --workload sweep (3 = the headline LLaMA-2-7B layer sweep)")
    ap.add_argument("--matrices", type=int, default=1 << 20, help="use only the first N matrices of the workload (debugging)")
    ap.add_argument("--overlap", type=int, default=0,
                    help="matrices decomposed concurrently (host threads, each with its own stream and workspace); "
                         "0 = 7 for workloads 2 and 3, 2 for workload 5 (52 GB of workspace per 8192x28672 matrix)")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel HIP-event pass")
    ap.add_argument("--grid", choices=("sweep36", "paper243"), default="sweep36",
                    help="workload 3 only: the 36-cell sweep the headline metric is quoted on, or the paper's own "
                         "243-cell search space (b0, b1 in {2,3,4}, b2 in {bf16,fp16,fp32}, B0 in {16,32,64}, "
                         "B1 in {16,64,256})")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one plain elementwise kernel that reads and writes exactly 1 GiB each, so that a "
                         "counter run (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) of this command holds a dispatch of "
                         "known HBM traffic to scale the counters by")
    ap.add_argument("--streams", type=int, default=None,
                    help="lq_svd_params.streams: interleaved sub-batches per matrix (0 = library default, 3, which is best "
                         "for one matrix at a time; default here: 2 with every matrix of a LLaMA-shaped layer in flight, "
                         "1 for workload 2, whose batches of 9 configurations are too small to split)")
    ap.add_argument("--gemm-mode", type=int, default=0, help="lq_svd_params.gemm_mode (0 = library default)")
    ap.add_argument("--first-width", type=int, default=0, help="lq_svd_params.first_width (0 = library default)")
    ap.add_argument("--workload", choices=("sweep", "quant", "matmul"), default="sweep")
    ap.add_argument("--tokens", type=int, default=4096, help="rows of X for --workload matmul")
    ap.add_argument("--precision", type=int, default=0, help="lq_matmul precision for --workload matmul (0 split, 1 bf16)")
    ap.add_argument("--hw-queues", type=int, default=None,
                    help="HIP hardware queues of this process (GPU_MAX_HW_QUEUES, 1..32).  Default 8 for the sweeps of "
                         "workloads 3 and 5, the runtime's own 4 otherwise.  Workload 3 keeps up to 14 streams busy (7 "
                         "matrices x 2 sub-batches); with 4 queues the streams share queues and a latency-bound "
                         "single-workgroup kernel (Cholesky, Jacobi) of one stream holds back the machine-filling kernels "
                         "of another in the same queue: 8 measured 4 %% faster, 14 no better.  Workload 2 (small "
                         "matrices, every kernel latency-bound) measured 16 %% slower with 8 than with 4")
    args = ap.parse_args()
    if args.hw_queues is None:
        args.hw_queues = 8 if (args.workload == "sweep" and args.config in (3, 5)) else 4
    if not 1 <= args.hw_queues <= 32:
        ap.error("--hw-queues must be within 1..32")
    os.environ["GPU_MAX_HW_QUEUES"] = str(args.hw_queues)       # read by the HIP runtime when it starts: before torch
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (several GPUs would share the sweep by matrix, "
              "without any collective; that path is not built).", file=sys.stderr)
        return 2
    if args.steps is None:
        args.steps = {"matmul": 100, "quant": 10}.get(args.workload) or {1: 50, 2: 2, 3: 2, 4: 5, 5: 1}[args.config]
    if args.warmup is None:
        args.warmup = {"matmul": 20, "quant": 2}.get(args.workload) or {1: 5, 2: 1, 3: 1, 4: 1, 5: 1}[args.config]

    if args.streams is None:
        args.streams = 1 if (args.workload == "sweep" and args.config == 2) else 2

    import torch
    from paper_2311_12023_amd import gen, lq

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    if args.workload == "matmul":
        if args.matrices > 7:
            args.matrices = 7
        return bench_matmul(args, torch, gen, lq, dev)
    if args.workload == "quant":
        return bench_quant(args, torch, gen, lq, dev)
    return bench_sweep(args, torch, gen, lq, dev)


if __name__ == "__main__":
    sys.exit(main())
