#!/usr/bin/env python3
"""Benchmark of the SKIM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

One step = one pass of the hot path over the metric layer (LLaMA-7B down-projection
shape, 4096 x 11008 fp32, synthetic): error table for b = 1..4 (30 Lloyd iterations)
-> greedy allocation to 3.2 average bits (on the device) -> selection of the allocated
clusterings -> packing (codes + fp16 codebooks).  Nothing inside a step waits for the host.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line: rows/s of the step, the
roofline figures of the dominant kernel (algorithmic lane-operations per launch over the kernel's time
from HIP events on its stream), the oracle's rate on the host cores, and figures of the other entry points.
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

N_ROWS, M_COLS = 4096, 11008
AVG_BITS = 3.2
ITERS = 30
HBM_PEAK_GBS = 8000.0
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: one non-packed 32-bit VALU lane-operation per lane per clock
ALU_PEAK_TLANEOPS = 256 * 4 * 16 * 2.4e9 / 1e12
MFMA_F32_PEAK_TFLOPS = 157.3


def alg_lane_ops_per_row(m: int) -> float:
    """Comparison-sort lower bound of the sorted formulation: m*log2(m) compare-exchanges of
    (key, payload) pairs at 5 VALU lane-operations each (compare + 4 selects)."""
    import math

    return 5.0 * m * math.log2(m)


def read_traffic():
    """HBM bytes per launch of the clustering kernel from the committed rocprofv3 counter summary."""
    p = os.path.join(ROOT, "profiles", "error_table_4096x11008_hbm_traffic.txt")
    try:
        for line in open(p):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


COUNTER_PASSES = (("FETCH_SIZE",), ("WRITE_SIZE",),
                  ("SQ_BUSY_CYCLES", "SQ_INSTS_VALU", "SQ_ACTIVE_INST_VALU", "SQ_INSTS_LDS", "SQ_ACTIVE_INST_LDS"))


def counter_child():
    """What a rocprofv3 counter pass runs: the plain copy of known size that calibrates the byte counters, then
    the error-table call on the metric layer a few times.  Prints nothing."""
    import torch

    import paper_2412_04180_amd as skim
    import skim_synth

    ctx = skim.Context(0)
    W_h, S_h = skim_synth.make_ws(2, 2)
    W, S = torch.from_numpy(W_h).cuda(), torch.from_numpy(S_h).cuda()
    dst = torch.empty_like(W)
    for _ in range(3):
        torch.mul(W, 1.0, out=dst)
    out = None
    for _ in range(3):
        out = ctx.error_table(W, S, iters=ITERS, out=out)
    torch.cuda.synchronize()


def collect_counters(timeout_s=150):
    """rocprofv3 --pmc over `bench.py --counter-child`, one run per counter group.  Returns
    {kernel: {counter: median value per dispatch}} with kernels 'copy', 'sort', 'lloyd', 'finish', or raises."""
    import csv
    import glob
    import shutil
    import statistics
    import subprocess
    import tempfile

    if shutil.which("rocprofv3") is None:
        raise RuntimeError("rocprofv3 not on PATH")
    res = {}
    for group in COUNTER_PASSES:
        d = tempfile.mkdtemp(prefix="skim_pmc_", dir="/tmp")
        try:
            cmd = ["timeout", "-s", "KILL", str(timeout_s), "rocprofv3", "--pmc", *group, "--kernel-trace",
                   "--output-format", "csv", "-d", d, "--", sys.executable, os.path.join(ROOT, "bench.py"),
                   "--counter-child"]
            r = subprocess.run(cmd, cwd="/tmp", env=dict(os.environ, TMPDIR="/tmp"), stdout=subprocess.PIPE,
                               stderr=subprocess.STDOUT, text=True)
            files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
            if r.returncode != 0 or not files:
                raise RuntimeError(f"rocprofv3 --pmc {' '.join(group)} failed (rc {r.returncode}): {r.stdout[-300:]}")
            vals = {}
            for row in csv.DictReader(open(files[0])):
                name = row["Kernel_Name"]
                kern = ("sort" if "sort_kernel" in name else "lloyd" if "lloyd_iter_kernel" in name else
                        "finish" if "finish_kernel" in name else "copy" if "elementwise" in name else None)
                if kern:
                    vals.setdefault((kern, row["Counter_Name"]), []).append(float(row["Counter_Value"]))
            for (kern, cname), v in vals.items():
                res.setdefault(kern, {})[cname] = statistics.median(v)
        finally:
            shutil.rmtree(d, ignore_errors=True)
    for k in ("copy", "sort", "lloyd", "finish"):
        if k not in res:
            raise RuntimeError(f"no dispatch of the {k} kernel in the counter output")
    return res


def host_cpus():
    """(logical CPUs this process may use, physical cores of the machine) from the OS."""
    try:
        logical = len(os.sched_getaffinity(0))
    except AttributeError:
        logical = os.cpu_count() or 1
    cores = set()
    try:
        phys = core = None
        for line in open("/proc/cpuinfo"):
            if line.startswith("physical id"):
                phys = line.split(":")[1].strip()
            elif line.startswith("core id"):
                core = line.split(":")[1].strip()
            elif not line.strip():
                if phys is not None and core is not None:
                    cores.add((phys, core))
                phys = core = None
    except OSError:
        pass
    return logical, (len(cores) or None)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-scale-loop", action="store_true")
    ap.add_argument("--no-other-shapes", action="store_true", help="skip the error-table timings on the other matrix shapes")
    ap.add_argument("--no-yardsticks", action="store_true", help="skip the exact-optimum yardsticks (extra figures only)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain elementwise copy of the W matrix (reads and writes n*m*4 bytes): "
                         "the known-size kernel that calibrates the HBM byte counters of a rocprofv3 --pmc run")
    ap.add_argument("--no-counters", action="store_true",
                    help="skip the rocprofv3 counter passes (HBM traffic, executed VALU instructions); the figures "
                         "are then taken from the committed summary under profiles/")
    ap.add_argument("--counter-child", action="store_true", help=argparse.SUPPRESS)
    args = ap.parse_args()
    if args.counter_child:
        counter_child()
        return
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no sharding or collectives are part of it)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2412_04180_amd as skim
    import skim_synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(2)

    ctx = skim.Context(0)
    stream = ctx.stream
    n, m = N_ROWS, M_COLS
    W_h, S_h = skim_synth.make_ws(2, 2)           # config 2, third matrix: 4096 x 11008
    assert W_h.shape == (n, m)
    W = torch.from_numpy(W_h).cuda()
    S = torch.from_numpy(S_h).cuda()

    table = dict(E=ctx.empty((n, 4), torch.float64), centroids_all=ctx.empty((n, 30), torch.float64),
                 upper_all=ctx.empty((n, 30), torch.float32))
    alloc = dict(bits=ctx.empty((n,), torch.uint8), info=ctx.empty((10,), torch.int64))
    sel = dict(centroids=ctx.empty((n, 16), torch.float64), upper=ctx.empty((n, 16), torch.float32))
    pk = dict(codes=ctx.empty((n * ((m * 4 + 31) // 32),), torch.int32), group_word_offset=ctx.empty((6,), torch.int64),
              row_perm=ctx.empty((n,), torch.int32), codebooks=ctx.empty((n * 16,), torch.int16))   # sized for 4 bits everywhere
    ctx.ensure_workspace(n, m)

    ev_a = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev_b = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev_c = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    ev_d = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    t_sort, t_lloyd = [0.0], [0.0]

    def step(i=None):
        if i is not None:
            ev_a[i].record(stream)
        ctx.error_table(W, S, iters=ITERS, out=table)
        if i is not None:
            ev_b[i].record(stream)
        ctx.greedy_allocate_device(table["E"], AVG_BITS, out=alloc)
        if i is not None:
            ev_c[i].record(stream)
        ctx.select_allocated(alloc["bits"], table, out=sel)
        ctx.pack(W, alloc["bits"], sel["centroids"], sel["upper"], out=pk)
        if i is not None:
            ev_d[i].record(stream)

    if args.copy_probe:
        probe_dst = torch.empty_like(W)
        for _ in range(3):
            torch.mul(W, 1.0, out=probe_dst)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # per-kernel times of the clustering call (the library keeps the events of its last call): a few
    # more calls, each read back before the next
    prof_calls = min(args.steps, 10)
    ctx.profile_enable(True)     # HIP events around the kernels of the clustering call, on its stream (after the timed region)
    for _ in range(prof_calls):
        ctx.error_table(W, S, iters=ITERS, out=table)
        stream.synchronize()
        a_, b_ = ctx.profile_last()
        t_sort[0] += a_
        t_lloyd[0] += b_
    total_s = t1 - t0
    ms_per_step = total_s / args.steps * 1e3
    ms_table = sum(a.elapsed_time(b) for a, b in zip(ev_a, ev_b)) / args.steps
    ms_pack = sum(a.elapsed_time(b) for a, b in zip(ev_c, ev_d)) / args.steps
    ms_alloc = sum(a.elapsed_time(b) for a, b in zip(ev_b, ev_c)) / args.steps
    info = alloc["info"].cpu().numpy()
    bits = alloc["bits"].cpu().numpy()
    spent, budget = int(info[8]), int(info[9])
    # the host allocator on the same table, for reference (not part of the step)
    E_h = table["E"].cpu().numpy()
    th0 = time.perf_counter()
    bits_h, _, _ = skim.greedy_allocate(E_h, AVG_BITS)
    ms_alloc_host = (time.perf_counter() - th0) * 1e3
    assert np.array_equal(bits, bits_h)
    ms_sort = t_sort[0] / prof_calls
    ms_lloyd = t_lloyd[0] / prof_calls

    rows_per_s = n / (ms_per_step * 1e-3)
    alg_ops = alg_lane_ops_per_row(m) * n
    achieved_alu = alg_ops / (ms_sort * 1e-3) / 1e12
    alg_bytes = 8.0 * n * m
    hbm_gbs = alg_bytes / (ms_sort * 1e-3) / 1e9
    # the same bound counted with what this kernel's compare-exchange costs (two instructions: fp64 min and max):
    # the comparison work then needs less time than reading W and S once, and HBM is the limiting roofline
    own_alu_us = 2.0 / 5.0 * alg_ops / (ALU_PEAK_TLANEOPS * 1e12) * 1e6
    hbm_floor_us = alg_bytes / (HBM_PEAK_GBS * 1e9) * 1e6
    roofline = {
        "bound": "alu", "kernel": "sort_kernel (dominant kernel of skim_error_table)",
        "achieved": round(achieved_alu, 4), "peak": round(ALU_PEAK_TLANEOPS, 2), "unit": "Tlaneop/s",
        "frac": round(achieved_alu / ALU_PEAK_TLANEOPS, 5),
        "traffic": None,
        "kernel_ms": round(ms_sort, 4),
        "algorithmic_lane_ops_per_launch": alg_ops,
        "algorithmic_lane_ops_basis": "m*log2(m) compare-exchanges per row at 5 lane-operations each (64-bit compare + 4 selects)",
        "hbm_algorithmic_bytes_per_launch": alg_bytes,
        "hbm_achieved_GBps": round(hbm_gbs, 1), "hbm_frac": round(hbm_gbs / HBM_PEAK_GBS, 5),
        "whole_table_frac": round(alg_ops / (ms_table * 1e-3) / 1e12 / ALU_PEAK_TLANEOPS, 5),
        "whole_table_hbm_frac": round(alg_bytes / (ms_table * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
        "counted_with_this_kernels_own_compare_exchange": {
            "lane_ops_per_compare_exchange": 2, "alu_floor_us": round(own_alu_us, 1), "hbm_floor_us": round(hbm_floor_us, 1),
            "limiting": "hbm" if hbm_floor_us > own_alu_us else "alu",
            "frac": round(max(hbm_floor_us, own_alu_us) / (ms_sort * 1e3), 5),
            "whole_table_frac": round(max(hbm_floor_us, own_alu_us) / (ms_table * 1e3), 5)},
    }

    out = {
        "metric": "rows/s for b=1..4 K-means error table, 4096x11008 fp32; % of roofline",
        "value": round(rows_per_s, 1), "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": "config 2, matrix 2: LLaMA-7B down_proj shape 4096x11008 fp32; error table b=1..4, "
                               "30 Lloyd iterations, greedy allocation to 3.2 bits, pack with fp16 codebooks",
                   "rows": n, "cols": m, "avg_bits": AVG_BITS, "iters": ITERS},
        "weights_per_s": round(rows_per_s * m, 1),
        "error_table_only_rows_per_s": round(n / (ms_table * 1e-3), 1),
        "breakdown_ms": {"error_table_call": round(ms_table, 4), "sort_kernel": round(ms_sort, 4),
                         "lloyd_kernel": round(ms_lloyd, 4), "greedy_device": round(ms_alloc, 4), "greedy_host_function_for_reference": round(ms_alloc_host, 4),
                         "select_and_pack": round(ms_pack, 4)},
        "allocation": {"spent": int(spent), "budget": int(budget),
                       "rows_per_bit": np.bincount(bits, minlength=5)[1:].tolist()},
        "roofline": roofline,
    }

    # consumer of the packed layout: codebook-lookup matrix-vector product over the packed layer
    xv = torch.randn(m, device="cuda")
    yv = ctx.dequant_matvec(pk, m, xv)
    torch.cuda.synchronize()
    mv0, mv1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    mv0.record(stream)
    for _ in range(10):
        ctx.dequant_matvec(pk, m, xv, out=yv)
    mv1.record(stream)
    torch.cuda.synchronize()
    mv_ms = mv0.elapsed_time(mv1) / 10
    used_words = int(pk["group_word_offset"].cpu().numpy()[5])
    packed_bytes = used_words * 4 + sum(int(info[b]) * (1 << b) for b in range(1, 5)) * 2
    out["dequant_matvec"] = {"ms": round(mv_ms, 4), "packed_bytes": int(packed_bytes),
                             "GBps": round(packed_bytes / (mv_ms * 1e-3) / 1e9, 1),
                             "frac_of_hbm_peak": round(packed_bytes / (mv_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
    yf = ctx.dequant_matvec_f32(pk, m, xv)
    torch.cuda.synchronize()
    mv0.record(stream)
    for _ in range(10):
        ctx.dequant_matvec_f32(pk, m, xv, out=yf)
    mv1.record(stream)
    torch.cuda.synchronize()
    mvf_ms = mv0.elapsed_time(mv1) / 10
    out["dequant_matvec_f32"] = {"ms": round(mvf_ms, 4), "packed_bytes": int(packed_bytes),
                                 "GBps": round(packed_bytes / (mvf_ms * 1e-3) / 1e9, 1),
                                 "frac_of_hbm_peak": round(packed_bytes / (mvf_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                 "max_abs_diff_to_float64_reader": float((yf.double() - yv).abs().max().item())}
    # yardsticks (not steps of the path): the least error any clustering / any allocation could reach
    E_d = table["E"]
    if not args.no_yardsticks:
        y0, y1, y2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        ctx.kmeans_optimal(W, S)
        ctx.dp_allocate(E_d, AVG_BITS)
        torch.cuda.synchronize()
        y0.record(stream)
        opt_d = ctx.kmeans_optimal(W, S)
        y1.record(stream)
        dp = ctx.dp_allocate(E_d, AVG_BITS)
        y2.record(stream)
        torch.cuda.synchronize()
        E_h = E_d.cpu().numpy()
        out["yardsticks"] = {
            "kmeans_optimal_ms": round(y0.elapsed_time(y1), 3),
            "lloyd_error_over_least_possible_per_bit_width": (E_h.sum(0) / opt_d.cpu().numpy().sum(0)).round(4).tolist(),
            "dp_allocate_ms": round(y1.elapsed_time(y2), 3),
            "greedy_error_over_optimal_allocation": round(float(E_h[np.arange(n), bits - 1].sum() / dp["info"][0].item()), 6),
        }
    if not args.no_other_shapes:
        out["error_table_other_shapes"] = bench_other_shapes(ctx, torch)
    if not args.no_scale_loop:
        out["scale_loop"] = bench_scale_loop(ctx, torch, np, skim_synth)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(W_h, S_h, np)
    # hardware counters of the clustering kernels, from rocprofv3 passes over a child process of this script
    counters, note = None, None
    if not args.no_counters:
        try:
            counters = collect_counters()
        except Exception as e:   # the bench line must not depend on the profiler
            note = f"live counter passes failed ({str(e)[:200]})"
    rf = out["roofline"]
    if counters is not None:
        copy_bytes = float(n) * m * 4
        ff = copy_bytes / counters["copy"]["FETCH_SIZE"]      # bytes per counter unit, from the copy of known size
        wf = copy_bytes / counters["copy"]["WRITE_SIZE"]
        byt = {k: counters[k]["FETCH_SIZE"] * ff + counters[k]["WRITE_SIZE"] * wf for k in ("sort", "lloyd", "finish")}
        c = counters["sort"]
        rf["traffic"] = round(byt["sort"])
        rf["traffic_source"] = ("rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes of this run (median per dispatch), "
                                "scaled by a plain copy of n*m*4 bytes")
        rf["traffic_read_write"] = [round(c["FETCH_SIZE"] * ff), round(c["WRITE_SIZE"] * wf)]
        rf["traffic_over_algorithmic"] = round(byt["sort"] / alg_bytes, 3)
        rf["whole_table_traffic"] = round(sum(byt.values()))
        rf["whole_table_traffic_over_algorithmic"] = round(sum(byt.values()) / alg_bytes, 3)
        rf["executed_lane_ops"] = round(c["SQ_INSTS_VALU"] * 64)
        rf["algorithmic_efficiency"] = round(alg_ops / (c["SQ_INSTS_VALU"] * 64), 4)
        # SQ_BUSY_CYCLES counts per shader engine (32); SQ_ACTIVE_INST_* in units of 4 clocks of one of 1024 SIMDs
        clocks = c["SQ_BUSY_CYCLES"] / 32.0
        rf["valu_busy"] = round(c["SQ_ACTIVE_INST_VALU"] * 4 / (clocks * 1024), 4)
        rf["lds_busy"] = round(c["SQ_ACTIVE_INST_LDS"] * 4 / (clocks * 1024), 4)
        cl = counters["lloyd"]
        rf["lloyd_kernel"] = {"executed_lane_ops": round(cl["SQ_INSTS_VALU"] * 64),
                              "valu_busy": round(cl["SQ_ACTIVE_INST_VALU"] * 4 / (cl["SQ_BUSY_CYCLES"] / 32.0 * 1024), 4),
                              "traffic": round(byt["lloyd"])}
    else:
        rf["traffic"] = read_traffic()
        rf["traffic_source"] = "profiles/error_table_4096x11008_hbm_traffic.txt (committed summary)" + (f"; {note}" if note else "")
    print(json.dumps(out))


def bench_other_shapes(ctx, torch, reps=3):
    """The error-table call on the other matrix shapes of the workload configs (values drawn on the device: normal
    weights, squared-normal sensitivities; timing only), and on the metric shape with weights that were rounded to
    float16 / bfloat16 first, as the weights of a released model are (every value then occurs many times in a row)."""
    res = []
    gen = torch.Generator(device="cuda").manual_seed(1)
    for n, m, fmt in ((4096, 4096, None), (11008, 4096, None), (22016, 8192, None), (8192, 22016, None),
                      (4096, 11008, "float16"), (4096, 11008, "bfloat16")):
        W = torch.randn(n, m, device="cuda", generator=gen) * 0.02
        if fmt is not None:
            W = W.to(getattr(torch, fmt)).float()
        S = torch.randn(n, m, device="cuda", generator=gen) ** 2
        out = ctx.error_table(W, S, iters=ITERS)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            ctx.error_table(W, S, iters=ITERS, out=out)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / reps * 1e3
        so, ll = ctx.profile_last()
        entry = {"rows": n, "cols": m, "table_ms": round(ms, 4), "sort_ms": round(so, 4),
                 "iterations_ms": round(ll, 4), "Gweights_per_s": round(n * m / ms / 1e6, 1)}
        if fmt is not None:
            entry["weights_rounded_to"] = fmt
        res.append(entry)
        del W, S, out
    return res


def bench_scale_loop(ctx, torch, np, skim_synth, iters=3):
    """Config-3 shape (4096 x 4096, H 4096^2): one iteration = scale step (loss + gradient + Adam),
    re-clustering at 3 bits, layer loss.  H here is X^T X / N from 8192 synthetic activations."""
    n = m = 4096
    W_h, S_h = skim_synth.make_ws(3, 0)
    W, S = torch.from_numpy(W_h).cuda(), torch.from_numpy(S_h).cuda()
    N = 8192
    Xb = torch.cat([torch.from_numpy(x).cuda().to(torch.bfloat16) for x in skim_synth.make_x(3, N, m, chunk=4096)])
    H = ctx.hessian_from_activations(Xb)           # H = X^T X / N on bf16 MFMA
    del Xb
    # the same kernel at the size of the paper's calibration set: 131072 activation vectors
    Nbig = 131072
    Xbig = torch.randn((Nbig, m), device="cuda", dtype=torch.float32).to(torch.bfloat16)
    Hbig = ctx.hessian_from_activations(Xbig)
    torch.cuda.synchronize()
    eh0, eh1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    eh0.record(ctx.stream)
    ctx.hessian_from_activations(Xbig, out=Hbig)
    eh1.record(ctx.stream)
    torch.cuda.synchronize()
    t_h = eh0.elapsed_time(eh1)
    hess_nt = (m + 255) // 256
    hess_tiles_done, hess_tiles_all = hess_nt * (hess_nt + 1) // 2, hess_nt * hess_nt
    del Xbig, Hbig
    bits = torch.full((n,), 3, dtype=torch.uint8, device="cuda")
    alpha = torch.ones(m, device="cuda")
    am, av = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
    cr = ctx.cluster_rows(W, S, bits, alpha=alpha)
    ctx.ensure_workspace(n, m)
    ctx.scale_step(W, S, H, cr["labels"], alpha, am, av, 1)
    ctx.layer_loss(W, S, H, cr["labels"], alpha=alpha)
    torch.cuda.synchronize()
    e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
    t_step = t_cluster = t_loss = 0.0
    losses = []
    for it in range(iters):
        e[0].record(ctx.stream)
        o = ctx.scale_step(W, S, H, cr["labels"], alpha, am, av, it + 2)
        e[1].record(ctx.stream)
        cr = ctx.cluster_rows(W, S, bits, alpha=alpha, out=cr)
        e[2].record(ctx.stream)
        l = ctx.layer_loss(W, S, H, cr["labels"], alpha=alpha, want_row_loss=False)
        e[3].record(ctx.stream)
        torch.cuda.synchronize()
        t_step += e[0].elapsed_time(e[1])
        t_cluster += e[1].elapsed_time(e[2])
        t_loss += e[2].elapsed_time(e[3])
        losses.append(l["loss"].item())
    flops = 2.0 * n * m * m
    # layer-wise (L-full) error table of the same layer: clustering + one contraction per bit width
    lf = ctx.error_table_lfull(W, S, H)
    torch.cuda.synchronize()
    e[0].record(ctx.stream)
    ctx.error_table_lfull(W, S, H, out=lf)
    e[1].record(ctx.stream)
    torch.cuda.synchronize()
    t_lfull = e[0].elapsed_time(e[1])
    # Alg. 2 as one call: clustering + 120 optimiser steps + final loss
    a2 = torch.ones(m, device="cuda")
    m2, v2 = torch.zeros(m, device="cuda"), torch.zeros(m, device="cuda")
    e[2].record(ctx.stream)
    tr = ctx.train_scale(W, S, H, bits, a2, m2, v2, steps=120)
    e[3].record(ctx.stream)
    torch.cuda.synchronize()
    t_train = e[2].elapsed_time(e[3])
    trace = tr["loss_trace"].cpu().numpy()
    return {"workload": "4096x4096, H 4096^2, 3 bits", "scale_step_ms": round(t_step / iters, 4),
            "hessian_131072x4096_ms": round(t_h, 3),
            # 2 N m^2 flops of the full product per second; the kernel computes the tiles on and above the diagonal
            # only (136 of 256 tiles of 256 x 256 here) and mirrors them: the matrix cores execute the fraction below
            "hessian_tflops": round(2.0 * Nbig * m * m / (t_h * 1e-3) / 1e12, 1),
            "hessian_executed_fraction_of_full_product": round(hess_tiles_done / hess_tiles_all, 4),
            "hessian_executed_tflops": round(2.0 * Nbig * m * m * (hess_tiles_done / hess_tiles_all) / (t_h * 1e-3) / 1e12, 1),
            "hessian_frac_of_bf16_mfma_peak": round(2.0 * Nbig * m * m * (hess_tiles_done / hess_tiles_all) / (t_h * 1e-3) / 1e12 / 2500.0, 4),
            "train_scale_120_steps_ms": round(t_train, 3),
            "train_scale_loss_first_last": [float(trace[0]), float(trace[-1])],
            "lfull_error_table_ms": round(t_lfull, 4),
            "lfull_error_table_tflops": round(4 * flops / (t_lfull * 1e-3) / 1e12, 2),
            "recluster_ms": round(t_cluster / iters, 4), "layer_loss_ms": round(t_loss / iters, 4),
            # 2 n m^2 flops of the contraction per second of the whole layer-loss call.  The contraction runs on the
            # bf16 matrix cores with every float32 operand cut into three bfloat16 pieces (the six leading piece
            # products per k: float32-grade result): the matrix cores execute 6 x 2 n m^2 flops
            "layer_loss_tflops": round(flops / (t_loss / iters * 1e-3) / 1e12, 2),
            "layer_loss_executed_bf16_tflops": round(6 * flops / (t_loss / iters * 1e-3) / 1e12, 1),
            "mfma_bf16_peak_tflops": 2500.0,
            "layer_loss_frac_of_mfma_peak": round(6 * flops / (t_loss / iters * 1e-3) / 1e12 / 2500.0, 4),
            "mfma_f32_peak_tflops": MFMA_F32_PEAK_TFLOPS,
            "layer_loss_over_f32_mfma_peak": round(flops / (t_loss / iters * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS, 4),
            "loss_after_each_iteration": losses}


def cpu_baseline(W_h, S_h, np, target_s=12.0):
    """The fp64 oracle, as it stands, on the host cores of this machine, on the first R rows of the same
    matrix (R sized for about target_s seconds): error table b = 1..4, greedy, labels, pack."""
    import oracle

    n = W_h.shape[0]
    probe = 128
    t0 = time.perf_counter()
    oracle.error_table(W_h[:probe], S_h[:probe])
    rate = probe / (time.perf_counter() - t0)
    R = int(min(n, max(probe, rate * target_s * 0.75)))
    Ws, Ss = np.ascontiguousarray(W_h[:R]), np.ascontiguousarray(S_h[:R])
    t0 = time.perf_counter()
    tab = oracle.error_table(Ws, Ss)
    t_tab = time.perf_counter() - t0
    g = oracle.greedy(tab["E"], AVG_BITS)
    cr = oracle.cluster_rows(Ws, Ss, g["bits"])
    oracle.pack(Ws, g["bits"], cr["labels"], cr["centroids"])
    t_all = time.perf_counter() - t0
    logical, physical = host_cpus()
    return {"value": round(R / t_all, 2), "unit": "rows/s", "cores": oracle.num_threads(), "kind": "oracle",
            "host_logical_cpus_available": logical, "host_physical_cores": physical,
            "sample": f"first {R} of {n} rows of the same 4096x11008 matrix: error table b=1..4 (30 iterations), "
                      f"greedy 3.2 bits, labels at the allocated widths, pack",
            "error_table_only_rows_per_s": round(R / t_tab, 2), "seconds": round(t_all, 2)}


if __name__ == "__main__":
    main()
