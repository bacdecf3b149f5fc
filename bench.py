#!/usr/bin/env python3
"""Benchmark of the SpMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps 100] [--warmup 10] [--workload bcsr_gate_proj] [--also wcsr_zipf]

A step is one asp_spmm call (C-initialisation, tile-width choice and the SpMM kernel) on a handle whose
format conversion and task partition were done once up front, with A, B and C resident in HBM -- the
protocol of the paper's Section IV (10 warm-up + 100 timed launches, throughput 2*nnz*N/t with nnz of
the original matrix).  The conversion time is reported separately in the same JSON line.

Prints ONE JSON line.  `value` uses the wall-clock time of the K timed steps; `roofline.achieved` uses the
average duration of a launch from one pair of events on the launch stream around the same K steps.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # MI355X fp32 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# the paper's numbers (NVIDIA H100, other hardware: context only)
PAPER_CONTEXT = {
    "hardware": "NVIDIA H100",
    "wcsr_speedup_over_accspmm": 1.47, "wcsr_speedup_over_cusparse": 6.24,
    "bcsr_end_to_end_prefill_speedup_at_90pct": 2.66,
    "bcsr_gate_proj_kernel_speedup_over_dense_90pct_n16384": 1.92,
}


def _measured_traffic(workload):
    """(bytes per launch through L2's memory side, kernel they were counted on) from the committed rocprofv3 --pmc
    summary, if one exists for this workload.  A counted value, not measured in this run: the kernel's name travels
    with it, and a CPU test checks that the name still exists in the sources with these template arguments."""
    p = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(p):
        try:
            e = json.load(open(p)).get(workload, {})
            return e.get("bytes_per_launch"), e.get("kernel")
        except Exception:
            return None, None
    return None, None


_DENSE_MEMO = {}
SINGLE_LAUNCHES = True    # --no-single-launches switches the second pass off
WARMUP_MIN_MS = 60.0      # --warmup-min-ms


def _dense_normal(synth, rows, cols, dt, seed):
    """synth.dense_normal, keeping the last operand: the sweeps reuse one 1 GB operand for many matrices."""
    key = (rows, cols, dt, seed)
    if key not in _DENSE_MEMO:
        _DENSE_MEMO.clear()
        _DENSE_MEMO[key] = synth.dense_normal(rows, cols, dt, seed)
    return _DENSE_MEMO[key]


_CSR_MEMO = {}


def _workload(synth, name):
    """synth.workload, keeping the last matrix: "<name>_n<width>" variants reuse the matrix of "<name>"."""
    import re
    base = re.sub(r"_n\d+", "", name)
    if base not in _CSR_MEMO:
        _CSR_MEMO.clear()
        _CSR_MEMO[base] = synth.workload(base)
    w = list(_CSR_MEMO[base])
    if base != name:
        w[4] = synth.workload_width(name)
    return tuple(w)


def run_workload(name, steps, warmup, torch, asp, synth, with_cpu_baseline, cpu_seconds=15.0):
    import numpy as np

    t0 = time.time()
    # "<workload>_xt": the same matrix through the K-contiguous entry, Y[N x m] = X[N x k] x A^T
    xt = name.endswith("_xt")
    # "<workload>_rcm": the matrix goes through the library's Reverse Cuthill-McKee reordering first (Section IV-A)
    rcm = name.endswith("_rcm")
    a, fmt, b_row, b_col, N, dt, seedB = _workload(synth, name[:-3] if xt else name[:-4] if rcm else name)
    t_reorder = None
    if rcm:
        t1 = time.time()
        perm = asp.asp_rcm(a.m, a.row_ptr, a.col_idx)
        rp, ci, va = asp.asp_permute_csr(a.m, a.k, a.row_ptr, a.col_idx, a.values, dt, perm, perm)
        a = synth.Csr(a.m, a.k, rp, ci, va, dt)
        t_reorder = time.time() - t1
    # the dense operand: drawn on the host (numpy, seeded) up to 2^27 elements, beyond that on the device (torch
    # generator, seeded) -- a 1 GB operand takes a minute on the host; the oracle always gets the device's bits
    shape = (N, a.k) if xt else (a.k, N)
    on_device = shape[0] * shape[1] > (1 << 27)
    B = None if on_device else _dense_normal(synth, shape[0], shape[1], dt, seedB)
    t_gen = time.time() - t0
    spmm = asp.asp_spmm_xt if xt else asp.asp_spmm

    stream = torch.cuda.current_stream().cuda_stream
    t0 = time.time()
    h = asp.asp_create_from_csr(fmt, dt, b_row, b_col, a.m, a.k, a.row_ptr, a.col_idx, a.values)
    t_convert = time.time() - t0
    info = asp.asp_get_info(h)
    plan = asp.asp_plan_spmm(h, N)
    # scratch for the partial tiles of split WCSR windows (set-up, like the conversion): bf16 handles need it, fp32
    # handles run at the same speed with it and are bitwise reproducible; nothing is allocated for other handles
    asp.asp_reserve(h, N)

    if on_device:
        g = torch.Generator(device="cuda")
        g.manual_seed(seedB)
        Bd = torch.randn(shape, dtype=torch.bfloat16 if dt == "bf16" else torch.float32, device="cuda", generator=g)
        if dt == "bf16":
            Bd = Bd.view(torch.int16)
    else:
        Bd = torch.from_numpy(B.view(np.int16) if dt == "bf16" else B).cuda()
    Cd = torch.empty((N, a.m) if xt else (a.m, N), dtype=torch.int16 if dt == "bf16" else torch.float32, device="cuda")
    bp, cp = Bd.data_ptr(), Cd.data_ptr()

    # untimed warm-up: `warmup` calls, and at least WARMUP_MIN_MS of them -- the GPU takes about 30 ms under load to
    # reach the clocks it then holds (measured: the first ~100 launches of the 0.27 ms BCSR workload run 8 % slower
    # than all later ones, whatever the split between warm-up and timed calls)
    warm_run = 0
    t_w = time.perf_counter()
    while warm_run < warmup or (time.perf_counter() - t_w) * 1e3 < WARMUP_MIN_MS:
        spmm(h, bp, cp, N, stream)
        warm_run += 1
        if warm_run % 16 == 0:
            torch.cuda.synchronize()   # keeps the loop's clock honest: launches are asynchronous
    torch.cuda.synchronize()
    # the timed region: exactly `steps` calls back to back, bracketed by a synchronisation on both sides (wall
    # clock -> value) and by one pair of events on the launch stream (-> average duration of a launch)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    w0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        spmm(h, bp, cp, N, stream)
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - w0) * 1e3 / steps
    kern_ms = ev0.elapsed_time(ev1) / steps
    per = None
    if SINGLE_LAUNCHES:
        # a second, untimed pass with events around every call: single launches, each on an otherwise idle GPU
        starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        ends = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
        for i in range(steps):
            starts[i].record()
            spmm(h, bp, cp, N, stream)
            ends[i].record()
        torch.cuda.synchronize()
        per = np.array([s.elapsed_time(e) for s, e in zip(starts, ends)])

    flops_eff = 2.0 * a.nnz * N
    esz = 2 if dt == "bf16" else 4
    if fmt == "bcsr":
        # work per stored block: 2*b_row*b_col*N flop (Section II-C: zeros inside blocks are computed)
        flops_alg = 2.0 * info.n_units * b_row * b_col * N
        bytes_alg = info.n_units * b_row * b_col * esz + a.k * N * esz + a.m * N * esz
        peak = PEAK_BF16_TFLOPS if dt == "bf16" else PEAK_F32_TFLOPS
        roof = {"bound": "mfma", "achieved": flops_alg / (kern_ms * 1e-3) / 1e12, "peak": peak, "unit": "TFLOP/s",
                # the same launch against the other roof: compulsory bytes (A once, B once, C once) over the HBM peak
                "frac_of_hbm_roof": bytes_alg / (kern_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
        extra = {"stored_blocks": int(info.n_units), "algorithmic_bytes": int(bytes_alg),
                 "hbm_floor_ms": bytes_alg / (PEAK_HBM_GBS * 1e9) * 1e3,
                 "mfma_floor_ms": flops_alg / (peak * 1e12) * 1e3}
    else:
        wci = asp.asp_export(h, asp.ASP_ARR_COL_IDX)
        tasks = asp.asp_export(h, asp.ASP_ARR_TASKS)
        real_cols = int((wci >= 0).sum())
        split_windows = int(len(np.unique(tasks[tasks[:, 3] != 0, 0]))) if len(tasks) else 0
        # per packed column: b_row values + 1 index of A, one gathered B row; per window one C tile
        # (every task of a split window writes a fp32 partial tile that is read back once)
        split_tasks = int((tasks[:, 3] != 0).sum()) if len(tasks) else 0
        bytes_alg = (info.n_units * (b_row * esz + 4) + real_cols * N * esz + a.m * N * esz
                     + 2 * split_tasks * b_row * N * 4)
        roof = {"bound": "hbm", "achieved": bytes_alg / (kern_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s"}
        extra = {"packed_cols": int(info.n_units), "real_cols": real_cols, "tasks": int(info.n_tasks),
                 "split_windows": split_windows, "algorithmic_bytes": int(bytes_alg),
                 "mfma_flops_padded": 2.0 * info.n_units * b_row * N}
    roof["frac"] = roof["achieved"] / roof["peak"]
    if fmt == "bcsr" and dt == "bf16":
        # (counter evidence, not measured in this run: profiles/bench_default_pmc.txt)
        roof["limiter"] = ("the memory side shared by the compute units: 1.68e9 B per launch (2.2 x compulsory; the 4 MB L2 of an "
                           "XCD holds half of the 7.3 MB slab of B its workgroups share) at 6.5-6.7 TB/s; on half of the compute units "
                           "the same launch is 1.27 x slower, not 2 x; matrix cores busy 0.40 of the cycles")
    roof["traffic"], traffic_kernel = _measured_traffic(name)
    if traffic_kernel:
        roof["traffic_source"] = "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled), kernel " + traffic_kernel
    roof["kernel_ms_avg"] = kern_ms
    if per is not None:   # the second pass ran
        roof["single_launch_ms_median"] = float(np.median(per))
        roof["single_launch_ms_avg"] = float(per.mean())

    res = {
        "workload": name, "format": fmt, "dtype": dt, "b_row": b_row, "b_col": b_col, "m": a.m, "k": a.k, "N": N, "nnz": a.nnz,
        "fill_ratio": info.fill_ratio, "bn": plan.bn, "workgroups": int(plan.workgroups),
        "value": flops_eff / (wall_ms * 1e-3) / 1e9, "ms_per_step": wall_ms, "roofline": roof,
        "convert_s": t_convert, "generate_s": t_gen, "warmup_calls_run": warm_run,
        "dense_operand_drawn_on": "device" if on_device else "host", **extra,
    }
    if t_reorder is not None:
        res["reorder_s"] = t_reorder

    if with_cpu_baseline and fmt == "bcsr" and dt == "bf16" and not xt and a.m * a.k <= (1 << 28):
        # context, as in the paper's Section IV-D (kernel speedup over the dense product): the vendor library's dense
        # bf16 GEMM of the same shape on this machine, A densified with its zeros
        dense = np.zeros((a.m, a.k), dtype=np.uint16)
        rows = np.repeat(np.arange(a.m), np.diff(a.row_ptr))
        dense[rows, a.col_idx] = a.values
        Ad = torch.from_numpy(dense.view(np.int16)).cuda().view(torch.bfloat16)
        Bb = Bd.view(torch.bfloat16)
        for _ in range(3):
            torch.matmul(Ad, Bb)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            torch.matmul(Ad, Bb)
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / 10
        res["dense_gemm_context"] = {"library": "torch.matmul (bf16, vendor GEMM)", "ms": dense_ms,
                                     "TFLOP/s": 2.0 * a.m * a.k * N / (dense_ms * 1e-3) / 1e12,
                                     "spmm_speedup_over_dense": dense_ms / kern_ms}
        del Ad, dense

    if with_cpu_baseline:
        import oracle
        # bounded sample: the oracle on a slice of B's columns (column j of C needs column j of B only)
        probe = min(N, 16)

        def first_columns(n):   # the oracle's operand is k x n: the first n columns (xt: tokens) as the GPU has them
            sl = Bd[:n].T if xt else Bd[:, :n]
            h = sl.contiguous().cpu().numpy()
            return h.view(np.uint16) if dt == "bf16" else h
        # size the sample from probes: widen the probe until it runs for half a second (a 16-column probe is mostly
        # fixed cost and overestimates the time per column several times), then scale to the target
        while True:
            Bp = first_columns(probe)
            t0 = time.perf_counter()
            oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, dt, Bp)
            tp = time.perf_counter() - t0
            if tp >= 0.5 or probe >= N:
                break
            probe = min(N, probe * 8)
        ncols = int(max(probe, min(N, cpu_seconds / max(tp / probe, 1e-9))))
        ncols = max(16, ncols // 16 * 16) if N >= 16 else N
        Bs = first_columns(ncols)
        t0 = time.perf_counter()
        ref, S = oracle.spmm(a.m, a.k, a.row_ptr, a.col_idx, a.values, dt, Bs)
        tc = time.perf_counter() - t0
        got = Cd[:ncols].cpu().numpy().T if xt else Cd[:, :ncols].cpu().numpy()
        got = synth.to_f64(np.ascontiguousarray(got).view(np.uint16), "bf16") if dt == "bf16" else got.astype(np.float64)
        bound = 1e-2 * S + 1e-5 if dt == "bf16" else 1e-5 * S
        ok = bool(np.isfinite(got).all() and (np.abs(got - ref) <= bound).all())
        res["cpu_baseline"] = {"value": 2.0 * a.nnz * ncols / tc / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "seconds": tc,
                               "sample": "first %d of %d columns of B, all %d rows (fp64 CSR oracle, includes the "
                                         "|A||B| bound pass)" % (ncols, N, a.m),
                               "gpu_matches_oracle_on_sample": ok}
    asp.asp_destroy(h)
    del Bd, Cd
    torch.cuda.empty_cache()
    return res


# The CDNA4 ladder (each rung = the library with benchmarking switches set; the switches only ever select
# among kernels that are built and parity-tested) and the tile-width / tile-order sweeps, after the
# paper's feature-by-feature study (Sections III-A..III-F, Table II) and its tile-width study (Section IV-C).
ABLATION = [
    ("no matrix cores: fp32 multiply-adds on the vector ALU (the generic kernel of the K-contiguous entry)",
     {"ASP_BCSR_XT": "generic"}, {"workload_suffix": "_xt", "max_steps": 5}),
    ("MFMA, synchronous register-staged loads, one tile per workgroup, 128x256 tiles",
     {"ASP_BCSR_KERNEL": "regstage", "ASP_BCSR_BN": "256"}),
    ("+ direct-to-LDS ring, resident workgroups (2 per CU), static XCD-aware schedule, 128x256 tiles",
     {"ASP_BCSR_BN": "256"}),
    ("  same, tiles pulled from per-XCD atomic counters instead of the static schedule", {"ASP_BCSR_BN": "256", "ASP_BCSR_SCHEDULE": "atomic"}),
    ("  same, 128x128 tiles", {"ASP_BCSR_BN": "128"}),
    ("  same, 128x64 tiles", {"ASP_BCSR_BN": "64"}),
    ("+ 128x128 wave tiles, one wave per SIMD, hand-ordered issue, 128x512 tiles (default)", {}),
    ("  same on 128 of the 256 compute units", {"ASP_BCSR_WORKGROUPS": "128"}),
    ("  same on 64 of the 256 compute units", {"ASP_BCSR_WORKGROUPS": "64"}),
    ("  same, tiles dealt without regard to XCDs", {"ASP_BCSR_XCD_AWARE": "0"}),
    ("  same, 1 N-tile per group", {"ASP_BCSR_GROUP_N": "1"}),
    ("  same, 4 N-tiles per group", {"ASP_BCSR_GROUP_N": "4"}),
]


def run_ablation(args):
    import subprocess
    rows = []
    for entry in ABLATION:
        label, env = entry[0], entry[1]
        opt = entry[2] if len(entry) > 2 else {}
        e = dict(os.environ)
        e.update(env)
        steps = min(args.steps, opt.get("max_steps", args.steps))
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", args.workload + opt.get("workload_suffix", ""),
               "--also", "", "--no-cpu-baseline", "--no-single-launches", "--steps", str(steps),
               "--warmup", str(min(args.warmup, steps))]
        out = subprocess.run(cmd, env=e, capture_output=True, text=True, timeout=600)
        if out.returncode != 0:
            rows.append({"variant": label, "switches": env, "error": out.stderr[-300:]})
            continue
        d = json.loads(out.stdout.strip().splitlines()[-1])
        rows.append({"variant": label, "switches": env, "kernel_ms": d["roofline"]["kernel_ms_avg"],
                     "achieved_tflops": d["roofline"]["achieved"], "frac": d["roofline"]["frac"], "bn": d["config"]["bn"]})
    print(json.dumps({"ablation": rows, "workload": args.workload, "steps": args.steps}))


# Config 5 (8192 x 8192, geometric block-row lengths, N = 65536: every block size and sparsity) and config 4
# (band + 64 long rows, 2e6 rows) at both dense widths: measured points that are not bench lines.
SWEEP = ["bcsr_sweep_b%d_s%d" % (b, p) for b in (128, 64, 32) for p in (50, 75, 90, 95, 99)] + \
        ["wcsr_band_dense_rows", "wcsr_band_dense_rows_n256", "wcsr_band_dense_rows_bf16", "wcsr_band_dense_rows_n256_bf16"]


def run_sweep(args, torch, asp, synth):
    global SINGLE_LAUNCHES
    SINGLE_LAUNCHES = False
    rows = []
    for name in SWEEP:
        r = run_workload(name, args.steps, args.warmup, torch, asp, synth, False)
        roof = r["roofline"]
        rows.append({"workload": name, "b_row": r["b_row"], "N": r["N"], "nnz": r["nnz"], "bn": r["bn"],
                     "kernel_ms": roof["kernel_ms_avg"], "effective_gflops": r["value"], "bound": roof["bound"],
                     "achieved": roof["achieved"], "unit": roof["unit"], "frac": roof["frac"],
                     "algorithmic_bytes": r["algorithmic_bytes"], "convert_s": r["convert_s"]})
        print("sweep", name, "%.4f ms" % roof["kernel_ms_avg"], "%.1f %s" % (roof["achieved"], roof["unit"]),
              file=sys.stderr, flush=True)
    print(json.dumps({"sweep": rows, "steps": args.steps, "warmup": args.warmup}))


# The paper's kernel-level case study (Section IV-D, the table of gate_proj latencies): 18944 x 3584 bf16, randomly
# block-sparsified, four sparsity levels x four sequence lengths, against the dense product of the same shape.
# The last two numbers of a cell are what the paper prints for its kernel on its hardware (latency, speedup over the
# dense library call there): context, not a target.
CASE_STUDY_PAPER = {
    (80, 1024): (0.17, 1.46), (90, 1024): (0.14, 1.58), (95, 1024): (0.12, 1.89), (99, 1024): (0.09, 2.60),
    (80, 4096): (0.55, 1.57), (90, 4096): (0.44, 1.98), (95, 4096): (0.39, 2.18), (99, 4096): (0.28, 3.04),
    (80, 16384): (2.06, 1.59), (90, 16384): (1.70, 1.92), (95, 16384): (1.46, 2.24), (99, 16384): (1.05, 3.19),
    (80, 65536): (8.12, 1.67), (90, 65536): (6.69, 1.96), (95, 65536): (5.88, 2.23), (99, 65536): (4.21, 3.06),
}


def run_case_study_grid(args, torch, asp, synth):
    global SINGLE_LAUNCHES
    SINGLE_LAUNCHES = False
    M, K = 18944, 3584
    dense_ms = {}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    Ad = (torch.randn((M, K), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    for N in (1024, 4096, 16384, 65536):
        Bb = torch.randn((K, N), device="cuda", generator=gen).to(torch.bfloat16)
        t_w = time.perf_counter()
        while (time.perf_counter() - t_w) * 1e3 < WARMUP_MIN_MS:
            torch.matmul(Ad, Bb)
            torch.cuda.synchronize()
        reps = 50 if N <= 16384 else 10
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            torch.matmul(Ad, Bb)
        e1.record()
        torch.cuda.synchronize()
        dense_ms[N] = e0.elapsed_time(e1) / reps
        del Bb
    del Ad
    torch.cuda.empty_cache()
    rows = []
    for blk in (128, 64):
        for pct in (80, 90, 95, 99):
            for N in (1024, 4096, 16384, 65536):
                name = "bcsr_gate_proj" + ("" if pct == 90 else "_s%d" % pct) + ("" if blk == 128 else "_b%d" % blk) + \
                       ("" if N == 16384 else "_n%d" % N)
                steps = args.steps if N <= 16384 else max(10, args.steps // 4)
                r = run_workload(name, steps, min(args.warmup, steps), torch, asp, synth, False)
                ms = r["roofline"]["kernel_ms_avg"]
                paper = CASE_STUDY_PAPER[(pct, N)]
                rows.append({"workload": name, "block": blk, "sparsity_pct": pct, "N": N, "stored_blocks": r["stored_blocks"],
                             "bn": r["bn"], "kernel_ms": ms, "effective_TFLOP/s": r["value"] / 1e3,
                             "frac_of_mfma_peak": r["roofline"]["frac"], "dense_ms": dense_ms[N],
                             "speedup_over_dense": dense_ms[N] / ms,
                             "paper_kernel_latency": paper[0], "paper_speedup_over_dense": paper[1]})
                print("grid", name, "%.4f ms" % ms, "dense %.4f ms" % dense_ms[N], "x%.2f" % (dense_ms[N] / ms),
                      file=sys.stderr, flush=True)
                torch.cuda.empty_cache()
    print(json.dumps({"case_study_grid": rows, "dense": "torch.matmul (bf16, vendor GEMM) of 18944 x 3584 by 3584 x N",
                      "paper_context": "Section IV-D kernel-level table, other hardware, 64 x 64 blocks",
                      "steps": args.steps}))


def box_peaks(torch):
    """What this machine sustains, beside the published peaks: matrix-core rate of an MFMA-only loop (both dtypes) and
    the bandwidth of a plain 1 GiB device copy (read + write), of a 1 GiB fill (write only) and of a read-only stream over 1 GiB."""
    from paper_2604_17834_amd import measure   # probe kernels in a library of their own, not the product's
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.zeros(16, dtype=torch.float32, device="cuda")
    res = {}
    for dt, iters in (("bf16", 4000), ("f32", 2000)):
        measure.asp_probe_mfma(dt, 200, out.data_ptr(), stream)
        torch.cuda.synchronize()
        best = 0.0
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flop = measure.asp_probe_mfma(dt, iters, out.data_ptr(), stream)
            e1.record()
            torch.cuda.synchronize()
            best = max(best, flop / (e0.elapsed_time(e1) * 1e-3) / 1e12)
        res["mfma_%s_TFLOPs" % dt] = best
    x = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    y = torch.empty_like(x)
    for name, fn, nbytes in (("copy_GBs", lambda: y.copy_(x), 2 * x.numel() * 4), ("fill_GBs", lambda: y.fill_(1.0), x.numel() * 4),
                             ("read_GBs", lambda: measure.asp_probe_read(x.data_ptr(), x.numel() * 4, out.data_ptr(), stream), x.numel() * 4)):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            fn()
        e1.record()
        torch.cuda.synchronize()
        res[name] = nbytes * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return res


def run_memory_probe(torch):
    """Read-only streams over buffers of different sizes, each read 20 times back to back: what the memory side
    delivers when the data fits the XCDs' L2s (4 MB each), the 256 MB memory-side cache, or only HBM.  The dense
    operand of the headline workload (117 MB) is re-read several times per launch; this says from where."""
    from paper_2604_17834_amd import measure
    stream = torch.cuda.current_stream().cuda_stream
    out = torch.zeros(16, dtype=torch.float32, device="cuda")
    rows = []
    big = torch.ones(1 << 30, dtype=torch.float32, device="cuda")   # 4 GiB; smaller probes read a prefix
    for mb in (16, 64, 117, 192, 384, 1024, 4096):
        nbytes = mb << 20
        for _ in range(3):
            measure.asp_probe_read(big.data_ptr(), nbytes, out.data_ptr(), stream)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20 if mb <= 1024 else 5
        e0.record()
        for _ in range(reps):
            measure.asp_probe_read(big.data_ptr(), nbytes, out.data_ptr(), stream)
        e1.record()
        torch.cuda.synchronize()
        rows.append({"MiB": mb, "GB/s": nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9})
    print(json.dumps({"memory_probe": rows, "kernel": "read-only stream, 16-byte loads, 8 in flight per lane, 8 workgroups per CU"}))


def run_mlp_chain(args, torch, synth):
    """The three projections of the case study's feed-forward block, chained without transposes through the
    K-contiguous entry: G = X Wg^T, U = X Wu^T (18944 x 3584 weights), Y = G Wd^T (3584 x 18944); activations
    stay tokens x features.  The element-wise gate between them is not part of the sparse path and is left out."""
    import numpy as np
    from paper_2604_17834_amd.linear import SparseLinear

    N, hid, ffn = 16384, 3584, 18944
    layers = {}
    for name, (o, i, seed) in {"gate": (ffn, hid, 1002), "up": (ffn, hid, 1032), "down": (hid, ffn, 1012)}.items():
        w = synth.block_sparse_bernoulli(o, i, 128, 128, 0.90, seed=seed)
        layers[name] = (SparseLinear(o, i, w.row_ptr, w.col_idx, w.values), w.nnz)
    X = torch.from_numpy(synth.dense_normal(N, hid, "bf16", 1005).view(np.int16)).cuda()
    G = torch.empty((N, ffn), dtype=torch.int16, device="cuda")
    U = torch.empty((N, ffn), dtype=torch.int16, device="cuda")
    Y = torch.empty((N, hid), dtype=torch.int16, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        layers["gate"][0](X, G, stream)
        layers["up"][0](X, U, stream)
        layers["down"][0](G, Y, stream)
    warm_run, t_w = 0, time.perf_counter()   # at least --warmup steps and at least --warmup-min-ms (see run_workload)
    while warm_run < args.warmup or (time.perf_counter() - t_w) * 1e3 < WARMUP_MIN_MS:
        step()
        warm_run += 1
        if warm_run % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    flops = 2.0 * N * sum(nnz for _, nnz in layers.values())
    print(json.dumps({"mlp_chain": {"tokens": N, "hidden": hid, "ffn": ffn, "block": 128, "sparsity": 0.90,
                                    "ms_per_step": ms, "effective_GFLOP/s": flops / (ms * 1e-3) / 1e9,
                                    "steps": args.steps, "warmup_steps_run": warm_run,
                                    "entry": "asp_spmm_xt x 3 (gate, up, down)"}}))
    for lin, _ in layers.values():
        lin.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="bcsr_gate_proj")
    ap.add_argument("--also", default="wcsr_zipf,bcsr_gate_proj_b64,bcsr_gate_proj_f32,wcsr_zipf_bf16,bcsr_gate_proj_xt,"
                                      "bcsr_down_proj,bcsr_down_proj_n1024_xt,bcsr_down_proj_n4096_xt,"
                                      "wcsr_band_dense_rows,wcsr_band_dense_rows_n256,bcsr_sweep_b128_s90",
                    help="comma list of further workloads reported under 'also' ('' = none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-reference", action="store_true",
                    help="only run a plain 1 GiB device copy (3 launches): the kernel of known size against "
                         "which rocprofv3's FETCH_SIZE / WRITE_SIZE counters are scaled")
    ap.add_argument("--memory-probe", action="store_true",
                    help="read-only streams over 16 MiB .. 4 GiB, repeated: the rate from L2, the memory-side cache and HBM")
    ap.add_argument("--mlp-chain", action="store_true",
                    help="time gate, up and down projections of the feed-forward block chained through asp_spmm_xt")
    ap.add_argument("--warmup-min-ms", type=float, default=60.0,
                    help="the untimed warm-up runs at least --warmup calls and at least this long (0: calls only)")
    ap.add_argument("--no-single-launches", action="store_true",
                    help="skip the second, untimed pass that times the same number of calls one by one (events around "
                         "each: median and mean of single launches)")
    ap.add_argument("--sweep", action="store_true",
                    help="the long-prefill BCSR grid (block sizes x sparsities) and the band + long rows WCSR workload at "
                         "both widths: one JSON object, no CPU baseline")
    ap.add_argument("--case-study-grid", action="store_true",
                    help="the paper's kernel-level case study: gate_proj at 4 sparsity levels x 4 sequence lengths, "
                         "128- and 64-wide blocks, with the dense product beside each")
    ap.add_argument("--ablation", action="store_true",
                    help="run the BCSR workload once per kernel variant (child processes) and print one JSON object")
    args = ap.parse_args()
    global SINGLE_LAUNCHES, WARMUP_MIN_MS
    SINGLE_LAUNCHES = not args.no_single_launches
    WARMUP_MIN_MS = args.warmup_min_ms
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU by design (one MI355X, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    if args.ablation:
        run_ablation(args)
        return

    import torch
    from paper_2604_17834_amd import binding as asp
    from paper_2604_17834_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the SpMM path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.copy_reference:
        x = torch.ones(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB written per launch
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_reference_bytes_read": x.numel() * 4, "copy_reference_bytes_written": x.numel() * 4,
                          "launches": 3}))
        return
    asp.lib()  # raises when the HIP library has not been built
    if args.memory_probe:
        run_memory_probe(torch)
        return
    if args.mlp_chain:
        run_mlp_chain(args, torch, synth)
        return
    if args.sweep:
        run_sweep(args, torch, asp, synth)
        return
    if args.case_study_grid:
        run_case_study_grid(args, torch, asp, synth)
        return

    main_res = run_workload(args.workload, args.steps, args.warmup, torch, asp, synth, not args.no_cpu_baseline)
    also = []
    for name in [s for s in args.also.split(",") if s and s != args.workload]:
        also.append(run_workload(name, args.steps, args.warmup, torch, asp, synth, not args.no_cpu_baseline, cpu_seconds=4.0))

    box = box_peaks(torch)
    for r in [main_res] + also:
        roof = r["roofline"]
        if roof["bound"] == "mfma":
            roof["frac_of_box"] = roof["achieved"] / box["mfma_%s_TFLOPs" % r["dtype"]]
        else:   # the gather is nine tenths reads: against the read-only stream
            roof["frac_of_box"] = roof["achieved"] / box["read_GBs"]
    line = {
        # (`warmup` echoes the request; the untimed warm-up runs that many calls AND at least warmup_min_ms, the
        # number of calls it ran is warmup_calls_run)
        "metric": ("effective SpMM GFLOP/s (2*nnz*N/t), BCSR gate_proj 18944x3584 bf16 128x128 blocks 90% sparse, N=16384"
                   if args.workload == "bcsr_gate_proj" else "effective SpMM GFLOP/s (2*nnz*N/t)") +
                  "; untimed warm-up = max(warmup calls, %g ms): %d calls ran" % (args.warmup_min_ms, main_res["warmup_calls_run"]),
        "value": main_res["value"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "warmup_min_ms": args.warmup_min_ms, "warmup_calls_run": main_res["warmup_calls_run"],
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res["dtype"], "data": "synthetic",
        "config": {"workload": args.workload, **{k: main_res[k] for k in
                                                   ("format", "b_row", "b_col", "m", "k", "N", "nnz", "bn", "workgroups")}},
        "roofline": main_res["roofline"],
        "cpu_baseline": main_res.get("cpu_baseline"),
        "detail": {k: v for k, v in main_res.items() if k not in ("roofline", "cpu_baseline", "value", "ms_per_step")},
        "also": also,
        "box_measured_peaks": box,
        "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
