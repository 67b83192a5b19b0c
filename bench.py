#!/usr/bin/env python3
"""Benchmark: LQ error-table sweep of one LLaMA-2-7B-shaped layer on one MI355X.

One step = the whole hot path over the workload: for each of the 7 weight matrices of the layer
(4x 4096x4096, 2x 4096x11008, 1x 11008x4096; synthetic, see paper_2311_12023_amd/gen.py) one
lq_error_table call over the 36 configurations bits {2,3,4,8} x B0 {16,32,64} x B1 {16,64,256}, rank 64,
10 LQ iterations each.  Inputs are resident in HBM before the timed region.  Prints one JSON line.
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

RANK = 64
ITERS = 10
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def cpu_baseline(first_matrix: np.ndarray) -> dict:
    """The oracle, as it stands, timed on a bounded sample of the workload on the host cores."""
    from oracle import lq_oracle as O
    O.build()
    sample = np.ascontiguousarray(first_matrix[:1024, :1024])
    cfg = O.config(3, 64, 256)
    t0 = time.perf_counter()
    O.lq(sample, RANK, cfg, ITERS)
    dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count() or 1
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    return {"value": 1.0 / dt, "unit": "matrix-configs/s on the sample", "cores": cores, "kind": "oracle",
            "sample": "one 1024x1024 corner of matrix 0, rank 64, NF3 B0=64 B1=256, 10 iterations "
                      f"(exact Jacobi SVD each iteration); {dt:.1f} s. A full 4096x4096 cell costs about "
                      "4^3 = 64 times as much."}


TRAFFIC_TABLE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "llama7b_layer_sweep_hbm_traffic.md")
FORWARD_TRAFFIC_TABLE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "llama7b_layer_forward_kernel_stats.md")


def measured_traffic(name: str, table: str | None = None):
    """HBM-side bytes per launch of a kernel class (fetch + write) from the committed counter summary, averaged over
    the class's template variants weighted by launches; None when the summary does not list the kernel."""
    try:
        lines = open(table or TRAFFIC_TABLE).read().splitlines()
    except OSError:
        return None
    base = name.split("<")[0]
    want = name.replace(" ", "")
    tot = n = 0.0
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
        if name.startswith("wide_gemm_kernel"):
            hit = kern.startswith(want[:-1] + ",")          # the table's names carry one more template argument
        else:
            hit = kern.split("<")[0] == base
        if hit:
            launches = float(cells[1])
            tot += launches * (float(cells[2]) + float(cells[3])) * 1e6
            n += launches
    return tot / n if n else None


def roofline_of(name: str, ms: float, launches: int, work: float) -> dict:
    """Roofline entry for one kernel class from its summed HIP-event time and algorithmic work."""
    sec = ms * 1e-3
    common = {"kernel": name, "traffic": None, "launches": launches, "avg_us": 1e3 * ms / launches}
    if name.startswith("wide_gemm_kernel"):
        lt, _, _, prec = (int(t) for t in name[name.index("<") + 1:name.index(">")].split(","))
        if prec == 0:      # fp32 MFMA: work is flops
            ach = work / sec / 1e12
            return {**common, "bound": "mfma", "achieved": ach, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / PEAK_FP32_MFMA_TFLOPS}
        # split-bf16 mode: three bf16 MFMAs per product leave the kernel bound by streaming A (4 B per element,
        # 2*l flop per element)
        ach = work / (2.0 * 32 * lt) * 4.0 / sec / 1e9
        return {**common, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                "algorithmic_tflops": work / sec / 1e12}
    if name.startswith("lowrank_blockquant"):   # (2r + 10) flop per weight, ALU + MFMA; W is read from HBM once per batch
        ach = work / sec / 1e12
        return {**common, "bound": "alu", "achieved": ach, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": ach / PEAK_FP32_MFMA_TFLOPS}
    ach = work / sec / 1e9
    return {**common, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}


PEAK_BF16_MFMA_TFLOPS = 2500.0
NF4_DOUBLE_QUANT = (4, 64, 256, 8, "bf16")


def bench_matmul(args, torch, gen, lq, dev) -> int:
    """Forward products Y = X (Q + L1 L2) of one LLaMA-2-7B-shaped layer; one step = all 7 matrices."""
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default: 2 for the sweep, 100 forward steps)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps first (default: 1 / 20)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--matrices", type=int, default=7, help="use only the first N matrices of the layer (debugging)")
    ap.add_argument("--no-isolated", action="store_true",
                    help="skip the extra non-overlapped profiled step that gives per-kernel rooflines without contention")
    ap.add_argument("--overlap", type=int, default=7,
                    help="matrices decomposed concurrently (host threads, each with its own stream and workspace)")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel HIP-event timing")
    ap.add_argument("--grid", choices=("sweep36", "paper243"), default="sweep36",
                    help="configuration grid: the 36-cell sweep the headline metric is quoted on, or the paper's own "
                         "243-cell search space (b0, b1 in {2,3,4}, b2 in {bf16,fp16,fp32}, B0 in {16,32,64}, "
                         "B1 in {16,64,256})")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also launch one plain elementwise kernel that reads and writes exactly 1 GiB each, so that a "
                         "counter run (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) of this command holds a dispatch of "
                         "known HBM traffic to scale the counters by")
    ap.add_argument("--streams", type=int, default=2,
                    help="lq_svd_params.streams: interleaved sub-batches per matrix (0 = library default, 3, which is best "
                         "for one matrix at a time; with every matrix of the layer in flight 2 is enough)")
    ap.add_argument("--gemm-mode", type=int, default=0, help="lq_svd_params.gemm_mode (0 = library default)")
    ap.add_argument("--workload", choices=("sweep", "matmul"), default="sweep",
                    help="sweep: the error-table sweep (the headline metric).  matmul: the consumer of a decomposition, "
                         "Y = X (Q + L1 L2) with just-in-time dequantization, for the 7 matrices of the layer at "
                         "--tokens rows of X (NF4 with double quantization, rank 64); prints its own JSON line")
    ap.add_argument("--tokens", type=int, default=4096, help="rows of X for --workload matmul")
    ap.add_argument("--precision", type=int, default=0, help="lq_matmul precision for --workload matmul (0 split, 1 bf16)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (the sweep shards over GPUs by "
              "matrix without any collective, see DESIGN.md).", file=sys.stderr)
        return 2
    if args.steps is None:          # a forward step is a few milliseconds, a sweep step more than half a second
        args.steps = 100 if args.workload == "matmul" else 2
    if args.warmup is None:
        args.warmup = 20 if args.workload == "matmul" else 1

    import torch
    from paper_2311_12023_amd import gen, lq

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    dev = torch.device("cuda:0")
    if args.workload == "matmul":
        return bench_matmul(args, torch, gen, lq, dev)
    cfgs = [lq.config(*g) for g in (gen.paper_config_grid() if args.grid == "paper243" else gen.config_grid())]
    params = lq.SvdParams(streams=args.streams, gemm_mode=args.gemm_mode)
    host = [gen.workload_matrix(3, i) for i in range(min(args.matrices, len(gen.LLAMA2_7B_LAYER)))]
    mats = [torch.from_numpy(w).to(dev) for w in host]
    # one workspace per concurrent matrix, each large enough for every shape of the layer
    shapes = {tuple(m.shape) for m in mats}
    nthreads = max(1, min(args.overlap, len(mats)))
    workspaces = [max((lq.error_table_workspace(d, k, RANK, len(cfgs), params, device=dev) for d, k in shapes),
                      key=lambda t: t.numel()) for _ in range(nthreads)]
    streams = [torch.cuda.Stream(device=dev) for _ in range(nthreads)]
    order = sorted(range(len(mats)), key=lambda i: -mats[i].numel())      # largest first
    torch.cuda.synchronize()
    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.mul(src, 2.0, out=dst)          # one elementwise kernel: 1 GiB in, 1 GiB out
        torch.cuda.synchronize()
        del src, dst

    import queue
    import threading

    def step(nthreads=nthreads, params=params):
        """One pass of the whole hot path over the layer: every matrix, every configuration."""
        out = [None] * len(mats)
        todo = queue.SimpleQueue()
        for i in order:
            todo.put(i)
        errors = []

        def worker(tid):
            try:
                with torch.cuda.stream(streams[tid]):
                    while True:
                        try:
                            i = todo.get_nowait()
                        except queue.Empty:
                            return
                        out[i] = lq.error_table(mats[i], RANK, cfgs, ITERS, seed=1, params=params,
                                                workspace=workspaces[tid])
            except Exception as exc:      # surfaced after the join
                errors.append(exc)

        threads = [threading.Thread(target=worker, args=(t,)) for t in range(nthreads)]
        for th in threads:
            th.start()
        for th in threads:
            th.join()
        if errors:
            raise errors[0]
        return out

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if not args.no_profile:
        lq.profile_enable(True)
        lq.profile_reset()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = lq.profile_read() if not args.no_profile else {}
    lq.profile_enable(False)
    # Per-kernel durations in the timed region include contention between concurrent matrices and streams.  One more
    # pass, one matrix at a time on one stream, gives each kernel's duration with the GPU to itself.
    prof_iso = {}
    if not (args.no_isolated or args.no_profile):
        lq.profile_enable(True)
        lq.profile_reset()
        step(nthreads=1, params=lq.SvdParams(streams=1, gemm_mode=args.gemm_mode))
        torch.cuda.synchronize()
        prof_iso = lq.profile_read()
        lq.profile_enable(False)

    cells = len(mats) * len(cfgs)
    value = cells * args.steps / dt
    # dominant kernel = largest summed event time
    kernels = {}
    for name, (ms, n, work) in prof.items():
        kernels[name] = {"ms_total": round(ms, 3), "launches": n, "avg_us": round(1e3 * ms / n, 2),
                         "work_per_s": work / (ms * 1e-3) if ms > 0 else 0.0}
    roof = None
    if prof:
        dname, (dms, dn, dwork) = max(prof.items(), key=lambda kv: kv[1][0])
        roof = roofline_of(dname, dms, dn, dwork)
        # counter-measured traffic per launch; the summary was taken in the default launch configuration
        if len(mats) == len(gen.LLAMA2_7B_LAYER) and args.streams == 2:
            roof["traffic"] = measured_traffic(dname)
    line = {
        "metric": "matrix-configs decomposed/sec (LLaMA-2-7B layer sweep)", "value": value, "unit": "matrix-configs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "LLaMA-2-7B-shaped layer (4x4096x4096, 2x4096x11008, 1x11008x4096), rank 64, "
                               + ("36 configs (bits 2/3/4/8 x B0 16/32/64 x B1 16/64/256)" if args.grid == "sweep36" else
                                  "243 configs (b0, b1 in 2/3/4 x b2 in bf16/fp16/fp32 x B0 16/32/64 x B1 16/64/256)")
                               + ", 10 LQ iterations",
                   "matrices": len(mats), "configs": len(cfgs), "iters": ITERS, "rank": RANK,
                   "concurrent_matrices": nthreads},
        "roofline": roof,
        "roofline_note": "dominant kernel (largest summed HIP-event time) of the timed region; its launches overlap "
                         "with other streams there, see roofline_isolated for the same kernels run alone",
        "roofline_isolated": {n: roofline_of(n, ms, cnt, wk) for n, (ms, cnt, wk) in prof_iso.items()
                              if n.startswith(("wide_gemm", "lowrank", "residual")) and ms > 1.0},
        "kernels": kernels,
        "error_table_checksum": float(sum(np.sqrt(e).sum() for e, _ in res)),
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(host[0])
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
