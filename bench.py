#!/usr/bin/env python3
"""Benchmark of the Fallback-Quantization hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch: fq_quantize of
the activation X (block abs-max, INT8 codes, fallback decision, residual
quantization, compaction) followed by fq_gemm Y = X W^T on the INT8 matrix
cores with the fallback term.  The weight is quantized once before timing (its
cost is reported separately).  Inputs are resident in HBM when timing starts.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0     # MI355X dense INT8 MFMA peak (published), TOP/s
HBM_PEAK_GBS = 8000.0
GEMM_SOURCE = os.path.join(ROOT, "paper_2503_08040_amd", "csrc", "fq_gemm.hip")
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "gemm_quantize_cfg2_hbm_traffic.md")


def measured_gemm_traffic(workload_name):
    """HBM-side bytes per fq_gemm launch as measured with rocprofv3 (FETCH_SIZE, WRITE_SIZE,
    each scaled by what the same counter reads for a copy of known size): read from the
    committed profile summary, which records the workload and the SHA-256 of the kernel source
    it was measured on.  None when the kernel source has changed since (the figure would be
    stale) or the summary does not cover this workload."""
    import hashlib
    import re
    try:
        text = open(TRAFFIC_PROFILE).read()
        sha = hashlib.sha256(open(GEMM_SOURCE, "rb").read()).hexdigest()
    except OSError:
        return None
    m = re.search(r"^gemm_traffic: workload=(\S+) bytes_per_launch=(\d+) fq_gemm_hip_sha256=([0-9a-f]{64})\s*$",
                  text, flags=re.M)
    if not m or m.group(1) != workload_name or m.group(3) != sha:
        return None
    return int(m.group(2))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def make_workload(name):
    from paper_2503_08040_amd import synth
    if name == "cfg1":
        return synth.config1()
    if name == "cfg2":
        return synth.config2()
    if name == "cfg3":
        return synth.config3()
    if name.startswith("cfg5"):
        parts = name.split(":")
        frac = float(parts[1]) if len(parts) > 1 else 0.05
        placement = parts[2] if len(parts) > 2 else "random"
        return synth.config5(frac=frac, placement=placement)
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(wl, budget_s=15.0):
    """Times the CPU oracle (as it stands) on a bounded window of the same workload."""
    from oracle import fqo
    rows = min(wl.M, 4096)
    t0 = time.perf_counter()
    oa = fqo.quantize(wl.X[:rows], 128, fqo.CRIT_ABSMAX_GT, wl.theta)
    tq = time.perf_counter() - t0
    ob = fqo.quantize(wl.W, 128, fqo.CRIT_NONE, 0.0)
    # calibrate on a small window, then size the timed window to the budget
    cols = min(wl.N, 64)
    t0 = time.perf_counter()
    fqo.gemm(fqo.OP_NT, oa, ob, window=(0, rows, 0, cols))
    tc = time.perf_counter() - t0
    scale = max(1.0, min(budget_s / max(tc, 1e-3), wl.N / cols))
    cols2 = int(min(wl.N, cols * scale)) // 64 * 64 or cols
    t0 = time.perf_counter()
    c32, cb16 = fqo.gemm(fqo.OP_NT, oa, ob, window=(0, rows, 0, cols2), want_bf16=True)
    tg = time.perf_counter() - t0
    # quantizing these rows of X is shared by all N columns: charge the window's share
    tq_share = tq * cols2 / wl.N
    ops = 2.0 * rows * cols2 * wl.K
    info = {"value": ops / (tg + tq_share) / 1e12, "unit": "TOPS", "cores": fqo.num_threads(),
            "kind": "oracle",
            "sample": f"oracle fqo_quantize on X[0:{rows}] + fqo_gemm on the {rows}x{cols2} output "
                      f"window (K={wl.K}); {tg:.2f}s gemm + {tq_share:.3f}s quantize share"}
    return info, (rows, cols2), (c32[:rows, :cols2], cb16[:rows, :cols2])


def accuracy(wl, window, oracle_out, y, x, w, qw):
    """Errors on the output window the CPU oracle has just computed: the GPU result against the
    oracle (the parity bar: max |diff| / max |ref| <= 1e-3) and, against the exact binary64
    product of the same bf16 inputs, the GPU result with fallback, plain block INT8 without
    fallback, and the bf16 GEMM."""
    import torch
    import paper_2503_08040_amd as fq
    from paper_2503_08040_amd import synth
    rows, cols = window
    f64 = lambda bits: synth.bf16_bits_to_f32(bits).astype(np.float64)
    exact = f64(wl.X[:rows]) @ f64(wl.W[:cols]).T
    ref_max, ref_norm = np.abs(exact).max(), np.linalg.norm(exact)

    def errs(c):
        d = c.astype(np.float64) - exact
        return {"max_over_max": float(np.abs(d).max() / ref_max),
                "frobenius": float(np.linalg.norm(d) / ref_norm)}

    got = y[:rows, :cols].float().cpu().numpy()
    ref = synth.bf16_bits_to_f32(oracle_out[1]) if y.dtype == torch.bfloat16 else oracle_out[0]
    qn = fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, capacity=0)
    plain = fq.fq_gemm(fq.FQ_OP_NT, qn, qw, out_dtype=y.dtype)[:rows, :cols].float().cpu().numpy()
    bf16 = torch.matmul(x[:rows], w[:cols].t()).float().cpu().numpy()
    return {"window": f"rows 0:{rows}, columns 0:{cols}",
            "vs_oracle_max_over_max": float(np.abs(got - ref).max() / np.abs(ref).max()),
            "vs_oracle_identical": bool(np.array_equal(got, ref)),
            "vs_fp64": errs(got), "vs_fp64_block_int8_without_fallback": errs(plain),
            "vs_fp64_bf16_gemm": errs(bf16)}


def _time_loop(fn, seconds, iters):
    """Median-free simple timing: warm up for `seconds`, then time `iters` calls with events."""
    import torch
    t_w = time.perf_counter()
    while time.perf_counter() - t_w < seconds:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def criteria(args):
    """Quantizer time under each fallback selector of Sec. 4.4 on the workload's X, every one
    set to flag the same number of blocks (the workload's planted outlier blocks)."""
    import torch
    import paper_2503_08040_amd as fq
    wl = make_workload(args.workload)
    x = torch.from_numpy(wl.X.view(np.int16)).cuda().view(torch.bfloat16)
    M, K = wl.M, wl.K
    out = fq.QTensor(M, K)
    k = len(wl.flagged_blocks)
    nb = out.nbr * out.nbc
    rows = []

    def add(name, fn, bytes_per_elt):
        ms = _time_loop(fn, 0.5, 100)
        n = fq.fq_qtensor_check(out)
        nbytes = bytes_per_elt(n / nb) * M * K
        rows.append({"selector": name, "flagged": n, "ms": round(ms, 5),
                     "algorithmic_gbs": round(nbytes / ms / 1e6, 1),
                     "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)})

    add("none", lambda: fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, out=out), lambda f: 3.0)
    add("absmax > theta", lambda: fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta, out=out),
        lambda f: 3.0 + f)
    add(f"top-{k} absmax", lambda: fq.fq_quantize_topk(x, k, out=out), lambda f: 5.0 + f)
    # L1 threshold between the k-th and (k+1)-th largest block error, found by bisection on the count
    lo, hi = 0.0, 1e9
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        fq.fq_quantize(x, fq.FQ_CRIT_L1_GT, mid, out=out)
        if fq.fq_qtensor_check(out) > k:
            lo = mid
        else:
            hi = mid
    add("L1 > theta", lambda: fq.fq_quantize(x, fq.FQ_CRIT_L1_GT, hi, out=out), lambda f: 3.0 + f)
    return {"workload": wl.name + "_selectors", "rows": M, "cols": K, "blocks": nb, "selectors": rows}


def quantizer_sizes(args):
    """fq_quantize (abs-max threshold, 5 % of the blocks flagged at random, drawn on the device)
    over activation sizes: time, algorithmic GB/s at (3 + f) B per element, and the fixed cost
    and streaming rate of the least-squares line time = t0 + bytes / rate through the points."""
    import torch
    import paper_2503_08040_amd as fq
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    rows = []
    for M, K in ((2048, 4096), (4096, 4096), (8192, 4096), (8192, 8192), (8192, 11008), (16384, 8192)):
        x = torch.randn((M, K), device="cuda", generator=g, dtype=torch.float32)
        nbr, nbc = M // 128, K // 128
        pick = torch.randperm(nbr * nbc, device="cuda", generator=g)[: int(round(0.05 * nbr * nbc))]
        xb = x.view(nbr, 128, nbc, 128)
        xb[pick // nbc, 5, pick % nbc, 7] = 200.0          # one outlier per flagged block
        x = x.to(torch.bfloat16)
        out = fq.QTensor(M, K)
        ms = _time_loop(lambda: fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, 20.0, out=out), 0.3, 100)
        f = fq.fq_qtensor_check(out) / (nbr * nbc)
        nbytes = (3.0 + f) * M * K
        rows.append({"rows": M, "cols": K, "flagged_fraction": round(f, 4), "ms": round(ms, 5),
                     "algorithmic_gbs": round(nbytes / ms / 1e6, 1),
                     "frac_of_hbm_peak": round(nbytes / ms / 1e6 / HBM_PEAK_GBS, 4)})
        log(f"[quantizer-sizes] {rows[-1]}")
        del x, xb, out
    b = np.array([(3.0 + r["flagged_fraction"]) * r["rows"] * r["cols"] for r in rows])
    t = np.array([r["ms"] * 1e-3 for r in rows])
    slope, t0 = np.polyfit(b, t, 1)
    return {"workload": "fq_quantize over activation sizes, 5 % of the blocks flagged", "sizes": rows,
            "fit": {"fixed_us": round(t0 * 1e6, 2), "streaming_gbs": round(1.0 / slope / 1e9, 1)}}


def sweep(args):
    """Workload config 5 (the square problem): M = K = N = 8192, fallback fraction and placement swept."""
    import torch
    import paper_2503_08040_amd as fq
    from paper_2503_08040_amd import synth
    M = K = N = 8192
    ops = 2.0 * M * N * K
    rows = []
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    qx = fq.QTensor(M, K)
    qw = fq.QTensor(N, K, capacity=0)
    ms_bf16 = None
    for placement in ("random", "sequential"):
        for frac in (0.0, 0.01, 0.05, 0.2, 0.5, 1.0):
            if placement == "sequential" and frac in (0.0, 1.0):
                continue          # identical to the random placement
            log(f"[sweep] f={frac} {placement}")
            wl = synth.config5(frac=frac, placement=placement)
            x = torch.from_numpy(wl.X.view(np.int16)).cuda().view(torch.bfloat16)
            w = torch.from_numpy(wl.W.view(np.int16)).cuda().view(torch.bfloat16)
            fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, out=qw)
            fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta, out=qx)
            n_fb = fq.fq_qtensor_check(qx)
            ms_q = _time_loop(lambda: fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta, out=qx), 0.3, 50)
            ms_g = _time_loop(lambda: fq.fq_gemm(fq.FQ_OP_NT, qx, qw, out=y), 1.0, 50)
            if ms_bf16 is None:
                ms_bf16 = _time_loop(lambda: torch.matmul(x, w.t(), out=y), 1.0, 50)
            rows.append({"placement": placement, "f_target": frac, "f": n_fb / 4096.0,
                         "ms_quantize": round(ms_q, 4), "ms_gemm": round(ms_g, 4),
                         "tops_gemm": round(ops / ms_g / 1e9, 1),
                         "tops_quant_plus_gemm": round(ops / (ms_q + ms_g) / 1e9, 1)})
            del x, w
    t0 = next(r for r in rows if r["f_target"] == 0.0)
    for r in rows:
        r["gemm_overhead_vs_f0"] = round(r["ms_gemm"] / t0["ms_gemm"], 3)
        r["speedup_vs_bf16"] = round(ms_bf16 / (r["ms_quantize"] + r["ms_gemm"]), 3)
    # crossover: first fraction (random placement) at which quantize+gemm is slower than bf16
    rnd = [r for r in rows if r["placement"] == "random"]
    cross = None
    for a, b in zip(rnd, rnd[1:]):
        ta, tb = a["ms_quantize"] + a["ms_gemm"], b["ms_quantize"] + b["ms_gemm"]
        if ta <= ms_bf16 < tb:
            cross = a["f"] + (b["f"] - a["f"]) * (ms_bf16 - ta) / (tb - ta)
    return {"workload": "cfg5_square_8192", "bf16_gemm_ms": round(ms_bf16, 4),
            "bf16_tflops": round(ops / ms_bf16 / 1e9, 1), "rows": rows,
            "crossover_fraction_random": None if cross is None else round(cross, 3)}


def overhead_curve(seconds_per_point=0.4, iters=30):
    """The square problem of workload config 5 (M = K = N = 8192) at a few fallback fractions:
    GEMM time and overhead against f = 0, quantize time, and the fraction at which quantize +
    fallback GEMM stops being faster than the bf16 GEMM (Sec. 6.3, App. B), interpolated
    linearly between the measured points.  Inputs follow config 5's recipe but are drawn on the
    device (N(0,1); exactly round(f * 4096) blocks get one column x100; "random": blocks drawn
    uniformly, "sequential": packed into the fewest block-rows; theta = 10), so that the default
    run stays short; bench.py --sweep runs the full table on the host-generated inputs."""
    import torch
    import paper_2503_08040_amd as fq
    M = K = N = 8192
    nbr = nbc = M // 128
    ops = 2.0 * M * N * K
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    base = torch.randn((M, K), device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    w = torch.randn((N, K), device="cuda", generator=g, dtype=torch.float32).to(torch.bfloat16)
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    qx = fq.QTensor(M, K)
    qw = fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, capacity=0)
    ms_bf16 = _time_loop(lambda: torch.matmul(base, w.t(), out=y), seconds_per_point, iters)
    points = []
    for placement, frac in (("random", 0.0), ("random", 0.05), ("random", 0.2), ("sequential", 0.05)):
        n_fb = int(round(frac * nbr * nbc))
        ids = (torch.randperm(nbr * nbc, device="cuda", generator=g)[:n_fb] if placement == "random"
               else torch.arange(n_fb, device="cuda"))
        x = base.clone()
        if n_fb:
            bi, bk = ids // nbc, ids % nbc
            col = bk * 128 + torch.randint(0, 128, (n_fb,), device="cuda", generator=g)
            rows = (bi[:, None] * 128 + torch.arange(128, device="cuda")[None, :]).reshape(-1)
            cols = col[:, None].expand(n_fb, 128).reshape(-1)
            x[rows, cols] = (x[rows, cols].float() * 100.0).to(torch.bfloat16)
        fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, 10.0, out=qx)
        got = fq.fq_qtensor_check(qx)
        ms_q = _time_loop(lambda: fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, 10.0, out=qx), 0.1, iters)
        ms_g = _time_loop(lambda: fq.fq_gemm(fq.FQ_OP_NT, qx, qw, out=y), seconds_per_point, iters)
        points.append({"placement": placement, "f": round(got / (nbr * nbc), 4),
                       "ms_quantize": round(ms_q, 4), "ms_gemm": round(ms_g, 4),
                       "tops_quant_plus_gemm": round(ops / (ms_q + ms_g) / 1e9, 1)})
        del x
    t0 = points[0]["ms_gemm"]
    for pt in points:
        pt["gemm_overhead_vs_f0"] = round(pt["ms_gemm"] / t0, 3)
        pt["speedup_vs_bf16"] = round(ms_bf16 / (pt["ms_quantize"] + pt["ms_gemm"]), 3)
    rnd = [pt for pt in points if pt["placement"] == "random"]
    total = lambda pt: pt["ms_quantize"] + pt["ms_gemm"]
    if total(rnd[0]) > ms_bf16:
        cross = 0.0                      # slower than bf16 even without fallback
    else:
        cross = None                     # faster than bf16 at every measured fraction
        for a, b in zip(rnd, rnd[1:]):
            if total(a) <= ms_bf16 < total(b):
                cross = a["f"] + (b["f"] - a["f"]) * (ms_bf16 - total(a)) / (total(b) - total(a))
    return {"workload": "cfg5_square_8192 (device-drawn inputs)", "bf16_gemm_ms": round(ms_bf16, 4),
            "bf16_tflops": round(ops / ms_bf16 / 1e9, 1), "points": points,
            "crossover_fraction_random": None if cross is None else round(cross, 3),
            "crossover_note": "largest fallback fraction (random placement) at which quantize + "
                              "fallback GEMM is still as fast as the bf16 GEMM, linear between the "
                              "measured points; null: beyond the last measured fraction"}


def group_sweep(args):
    """Sec. 4.5 / Fig. 1b: throughput of the plain block-INT8 GEMM (Eq. (1), no fallback) over the
    quantization group size g in {32, 64, 128} on square problems, one kernel for all three
    (fq_gemm_plain), beside the tuned g = 128 kernel (fq_gemm) and the bf16 GEMM."""
    import torch
    import paper_2503_08040_amd as fq
    rows = []
    g_ = torch.Generator(device="cuda")
    g_.manual_seed(7)
    for n in (2048, 4096, 8192):
        x = torch.randn((n, n), device="cuda", generator=g_, dtype=torch.float32).to(torch.bfloat16)
        w = (torch.randn((n, n), device="cuda", generator=g_, dtype=torch.float32) * 0.02).to(torch.bfloat16)
        y = torch.empty((n, n), dtype=torch.bfloat16, device="cuda")
        ops = 2.0 * n * n * n
        row = {"M=K=N": n}
        for g in (32, 64, 128):
            qx = fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, capacity=0, block=g)
            qw = fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, capacity=0, block=g)
            ms = _time_loop(lambda: fq.fq_gemm_plain(fq.FQ_OP_NT, qx, qw, out=y), 0.5, 30)
            msq = _time_loop(lambda: fq.fq_quantize(x, fq.FQ_CRIT_NONE, 0.0, out=qx), 0.1, 30)
            row[f"plain_g{g}"] = {"ms_gemm": round(ms, 4), "tops": round(ops / ms / 1e9, 1),
                                  "ms_quantize": round(msq, 4)}
            if g == 128:
                ms = _time_loop(lambda: fq.fq_gemm(fq.FQ_OP_NT, qx, qw, out=y), 0.5, 30)
                row["tuned_g128"] = {"ms_gemm": round(ms, 4), "tops": round(ops / ms / 1e9, 1)}
            del qx, qw
        ms = _time_loop(lambda: torch.matmul(x, w.t(), out=y), 0.5, 30)
        row["bf16"] = {"ms_gemm": round(ms, 4), "tflops": round(ops / ms / 1e9, 1)}
        rows.append(row)
        log(f"[group-sweep] {row}")
    return {"workload": "square NT, plain block INT8 (no fallback), group size swept", "rows": rows}


def gemm_ablation(args):
    """Times fq_gemm on the workload with the library and with each ablation build of it (one
    component of the k-loop removed or added, see csrc/fq_gemm.hip), each in a process of its
    own because a process loads one build.  The ablation builds compute wrong products."""
    import subprocess
    from paper_2503_08040_amd import build as hip_build
    rows = []
    for name in ["library", "library_biased"] + list(hip_build.ABLATIONS):
        env = dict(os.environ)
        if not name.startswith("library"):
            path = hip_build.ablation_lib(name)
            if not os.path.exists(path):
                raise SystemExit(f"{path} is missing: python -m paper_2503_08040_amd.build")
            env["FQ_LIBRARY"] = path
        r = subprocess.run([sys.executable, os.path.abspath(__file__), "--gemm-only",
                            "--workload", args.workload, "--steps", str(args.steps)] +
                           (["--biased"] if name == "library_biased" else []),
                           capture_output=True, text=True, env=env, timeout=600)
        if r.returncode != 0:
            raise SystemExit(f"ablation {name} failed: {r.stderr[-2000:]}")
        row = json.loads(r.stdout.strip().splitlines()[-1])
        row["build"] = name
        rows.append(row)
        log(f"[gemm-ablation] {row}")
    base = rows[0]["ms_gemm"]
    for row in rows:
        row["vs_library"] = round(row["ms_gemm"] / base, 4)
    return {"workload": args.workload, "rows": rows}


def gemm_only(args):
    """fq_gemm alone on the workload: milliseconds per launch (HIP events, after a warm-up)."""
    import torch
    import paper_2503_08040_amd as fq
    wl = make_workload(args.workload)
    x = torch.from_numpy(wl.X.view(np.int16)).cuda().view(torch.bfloat16)
    w = torch.from_numpy(wl.W.view(np.int16)).cuda().view(torch.bfloat16)
    qx = fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta)
    qw = fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, capacity=0)
    y = torch.empty((wl.M, wl.N), dtype=torch.bfloat16, device="cuda")
    entry = fq.fq_gemm_biased if args.biased else fq.fq_gemm
    ms = _time_loop(lambda: entry(fq.FQ_OP_NT, qx, qw, out=y), 1.0, max(args.steps, 50))
    ops = 2.0 * wl.M * wl.N * wl.K
    return {"ms_gemm": round(ms, 4), "tops": round(ops / ms / 1e9, 1)}


def backward(args):
    """Sec. 5.1 / 5.3: dY is block-quantized with stochastic rounding, then two plain block GEMMs
    dX = dY W and dW = dY^T X_ctx (X_ctx: the stochastic block-INT8 context stored in forward)."""
    import torch
    import paper_2503_08040_amd as fq
    from paper_2503_08040_amd import synth
    wl = make_workload(args.workload)
    M, K, N = wl.M, wl.K, wl.N
    rng = np.random.default_rng(1)
    dy_bits = synth.to_bf16_bits((rng.standard_t(3.0, size=(M, N)) * 1e-3).astype(np.float32))
    dy = torch.from_numpy(dy_bits.view(np.int16)).cuda().view(torch.bfloat16)
    x = torch.from_numpy(wl.X.view(np.int16)).cuda().view(torch.bfloat16)
    w = torch.from_numpy(wl.W.view(np.int16)).cuda().view(torch.bfloat16)
    qdy = fq.QTensor(M, N, capacity=0, want_transposed=True)
    qw = fq.QTensor(N, K, capacity=0, want_transposed=True)
    qx = fq.QTensor(M, K, capacity=0, want_transposed=True)
    fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, out=qw)
    fq.fq_quantize_sr(x, 5, out=qx)
    dx = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    dw = torch.empty((N, K), dtype=torch.bfloat16, device="cuda")
    ms_q = _time_loop(lambda: fq.fq_quantize_sr(dy, 7, out=qdy), 0.5, 50)
    ms_dx = _time_loop(lambda: fq.fq_gemm(fq.FQ_OP_NN, qdy, qw, out=dx), 1.0, 50)
    ms_dw = _time_loop(lambda: fq.fq_gemm(fq.FQ_OP_TN, qdy, qx, out=dw), 1.0, 50)
    ms_bdx = _time_loop(lambda: torch.matmul(dy, w, out=dx), 1.0, 30)
    ms_bdw = _time_loop(lambda: torch.matmul(dy.t(), x, out=dw), 1.0, 30)
    ops = 2.0 * M * N * K
    return {"workload": wl.name + "_backward", "ms_quantize_sr_dY": round(ms_q, 4),
            "quantize_sr_gbs": round(4.0 * M * N / ms_q / 1e6, 1),
            "ms_gemm_dX": round(ms_dx, 4), "tops_dX": round(ops / ms_dx / 1e9, 1),
            "ms_gemm_dW": round(ms_dw, 4), "tops_dW": round(ops / ms_dw / 1e9, 1),
            "effective_tops": round(2 * ops / (ms_q + ms_dx + ms_dw) / 1e9, 1),
            "bf16_ms_dX": round(ms_bdx, 4), "bf16_ms_dW": round(ms_bdw, 4),
            "speedup_vs_bf16": round((ms_bdx + ms_bdw) / (ms_q + ms_dx + ms_dw), 3)}


def context(args):
    """Sec. 5.2 / 5.3: 1 x 128 group INT10 compression of a non-linear layer's activation context
    (the workload's X: for cfg3 the SiLU-GLU output fed to the down projection) and its
    dequantization, each against the HBM roofline."""
    import torch
    import paper_2503_08040_amd as fq
    wl = make_workload(args.workload)
    x = torch.from_numpy(wl.X.view(np.int16)).cuda().view(torch.bfloat16)
    rows, cols = x.shape
    packed, scales = fq.fq_ctx_quantize(x)
    back = torch.empty_like(x)
    ms_q = _time_loop(lambda: fq.fq_ctx_quantize(x, packed, scales), 1.0, 100)
    ms_d = _time_loop(lambda: fq.fq_ctx_dequantize(packed, scales, rows, cols, out=back), 1.0, 100)
    ms_c = _time_loop(lambda: back.copy_(x), 1.0, 100)
    nbytes = 2.0 * rows * cols + packed.numel() + 4.0 * scales.numel()
    return {"workload": wl.name + "_context_int10", "rows": rows, "cols": cols,
            "bytes_bf16": 2 * rows * cols, "bytes_int10": packed.numel() + 4 * scales.numel(),
            "ms_quantize": round(ms_q, 5), "ms_dequantize": round(ms_d, 5),
            "roofline_quantize": {"bound": "hbm", "achieved": round(nbytes / ms_q / 1e6, 1),
                                  "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                  "frac": round(nbytes / ms_q / 1e6 / HBM_PEAK_GBS, 4)},
            "roofline_dequantize": {"bound": "hbm", "achieved": round(nbytes / ms_d / 1e6, 1),
                                    "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                    "frac": round(nbytes / ms_d / 1e6 / HBM_PEAK_GBS, 4)},
            "bf16_copy_gbs": round(4.0 * rows * cols / ms_c / 1e6, 1),
            "glu": glu_times(x), "rmsnorm": rmsnorm_times(x)}


def rmsnorm_times(x):
    """RMS normalization forward / backward with a fused INT10 context on a tensor of x's shape:
    algorithmic bytes per element forward 2 (x) + 2 (y) + 1.28 (context) = 5.28, backward
    2 (dy) + 1.28 + 2 (dx) = 5.28 (the gain, rstd and the dw partial sums are negligible; the
    backward pass as built reads dy and the context twice, 8.56 in all)."""
    import torch
    import paper_2503_08040_amd as fq
    rows, cols = x.shape
    w = torch.ones(cols, dtype=torch.bfloat16, device=x.device)
    y, rstd, ctx = fq.fq_rmsnorm_forward(x, w, 1e-5)
    ms_f = _time_loop(lambda: fq.fq_rmsnorm_forward(x, w, 1e-5), 1.0, 50)
    ms_b = _time_loop(lambda: fq.fq_rmsnorm_backward(y, ctx, rstd, w, n_parts=256), 1.0, 50)
    nbytes = 4.0 * rows * cols + ctx[0].numel() + 4.0 * ctx[1].numel()
    return {"ms_forward": round(ms_f, 5), "ms_backward": round(ms_b, 5),
            "forward_gbs": round(nbytes / ms_f / 1e6, 1), "backward_gbs": round(nbytes / ms_b / 1e6, 1),
            "forward_frac_of_hbm_peak": round(nbytes / ms_f / 1e6 / HBM_PEAK_GBS, 4),
            "backward_frac_of_hbm_peak": round(nbytes / ms_b / 1e6 / HBM_PEAK_GBS, 4)}


def glu_times(x):
    """SiLU-GLU forward and backward with fused INT10 contexts on two tensors of x's shape
    (stand-ins for the gate and up projections): algorithmic bytes per element pair
    forward 4 (x1, x2) + 2 (y) + 2*1.28 (contexts) = 8.56, backward 2 (dy) + 2.56 + 4 = 8.56."""
    import torch
    import paper_2503_08040_amd as fq
    rows, cols = x.shape
    x2 = torch.roll(x, 1, 0).contiguous()
    y, c1, c2 = fq.fq_glu_forward(x, x2)
    ms_f = _time_loop(lambda: fq.fq_glu_forward(x, x2), 1.0, 50)
    ms_b = _time_loop(lambda: fq.fq_glu_backward(y, c1, c2), 1.0, 50)
    ctx_bytes = 2.0 * (c1[0].numel() + 4.0 * c1[1].numel())
    fwd_bytes = 6.0 * rows * cols + ctx_bytes
    bwd_bytes = 6.0 * rows * cols + ctx_bytes
    return {"ms_forward": round(ms_f, 5), "ms_backward": round(ms_b, 5),
            "forward_gbs": round(fwd_bytes / ms_f / 1e6, 1),
            "backward_gbs": round(bwd_bytes / ms_b / 1e6, 1),
            "forward_frac_of_hbm_peak": round(fwd_bytes / ms_f / 1e6 / HBM_PEAK_GBS, 4),
            "backward_frac_of_hbm_peak": round(bwd_bytes / ms_b / 1e6 / HBM_PEAK_GBS, 4)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg2",
                    help="cfg2 (default, GLU up/gate 4096x4096x11008), cfg3, cfg1, cfg5[:frac[:placement]]")
    ap.add_argument("--out-dtype", default="bf16", choices=["bf16", "f32"])
    ap.add_argument("--warmup-seconds", type=float, default=1.5,
                    help="minimum duration of the untimed warm-up (clock ramp)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bf16-baseline", action="store_true")
    ap.add_argument("--no-tolerance-variant", action="store_true",
                    help="skip timing fq_gemm_biased beside the exact kernel (about 2 s)")
    ap.add_argument("--sweep", action="store_true",
                    help="config-5 sweep (8192^3): fallback fraction x placement, overhead curve and "
                         "crossover against the bf16 GEMM; prints one JSON object with a table")
    ap.add_argument("--no-overhead-curve", action="store_true",
                    help="skip the compact config-5 overhead curve (about 10 s)")
    ap.add_argument("--pipeline-probe", action="store_true",
                    help="run the register-resident pipeline probe (cycles per unit and clock of the "
                         "MFMA + dequantization mix; about 15 s) and print its table as one JSON object")
    ap.add_argument("--quantizer-sizes", action="store_true",
                    help="time fq_quantize over activation sizes: fixed cost and streaming rate")
    ap.add_argument("--gemm-ablation", action="store_true",
                    help="time fq_gemm with each ablation build of the library (a component of the "
                         "k-loop removed or added); prints one JSON object with a table")
    ap.add_argument("--gemm-only", action="store_true",
                    help="time fq_gemm alone on the workload and print {ms_gemm, tops}")
    ap.add_argument("--biased", action="store_true",
                    help="with --gemm-only: time fq_gemm_biased, the tolerance variant, instead")
    ap.add_argument("--group-sweep", action="store_true",
                    help="Fig. 1b: plain block-INT8 GEMM at group sizes 32, 64, 128 on square problems")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the register-only MFMA throughput probe (about 3 s)")
    ap.add_argument("--backward", action="store_true",
                    help="time the paper's backward recipe on the workload's shape instead: "
                         "fq_quantize_sr(dY) + fq_gemm NN (dX) + fq_gemm TN (dW)")
    ap.add_argument("--context", action="store_true",
                    help="time the INT10 1x128 context compression / decompression of the "
                         "workload's X instead (GB/s against the HBM roofline)")
    ap.add_argument("--criteria", action="store_true",
                    help="time the quantizer under each fallback selector (threshold, top-k, L1) "
                         "on the workload's X instead")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain device copy of 1 GiB (5 times) and exit: gives the "
                         "profiler's FETCH_SIZE / WRITE_SIZE counters a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py measures one GPU: this build has no multi-GPU path "
                         "(run with --gpus 1)")

    import torch
    import paper_2503_08040_amd as fq

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4,
                          "calibrate_copy_bytes_written": src.numel() * 4}), flush=True)
        return
    if args.sweep:
        print(json.dumps(sweep(args)), flush=True)
        return
    if args.pipeline_probe:
        import subprocess
        tool = os.path.join(ROOT, "paper_2503_08040_amd", "pipeline_probe")
        r = subprocess.run([tool], capture_output=True, text=True, timeout=300)
        if r.returncode != 0:
            raise SystemExit(f"pipeline_probe failed: {r.stderr}")
        print(json.dumps({"tool": "pipeline_probe",
                          "modes": [json.loads(ln) for ln in r.stdout.splitlines() if ln.startswith("{")]}),
              flush=True)
        return
    if args.group_sweep:
        print(json.dumps(group_sweep(args)), flush=True)
        return
    if args.quantizer_sizes:
        print(json.dumps(quantizer_sizes(args)), flush=True)
        return
    if args.gemm_only:
        print(json.dumps(gemm_only(args)), flush=True)
        return
    if args.gemm_ablation:
        print(json.dumps(gemm_ablation(args)), flush=True)
        return
    if args.backward:
        print(json.dumps(backward(args)), flush=True)
        return
    if args.context:
        print(json.dumps(context(args)), flush=True)
        return
    if args.criteria:
        print(json.dumps(criteria(args)), flush=True)
        return
    log(f"[bench] generating {args.workload}")
    wl = make_workload(args.workload)
    M, K, N = wl.M, wl.K, wl.N
    x = torch.from_numpy(wl.X.view(np.int16)).cuda().view(torch.bfloat16)
    w = torch.from_numpy(wl.W.view(np.int16)).cuda().view(torch.bfloat16)
    out_dtype = torch.bfloat16 if args.out_dtype == "bf16" else torch.float32
    y = torch.empty((M, N), dtype=out_dtype, device="cuda")

    qx = fq.QTensor(M, K)
    qw = fq.QTensor(N, K, capacity=0)
    fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, out=qw)
    fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta, out=qx)
    n_fb = fq.fq_qtensor_check(qx)
    f = n_fb / (qx.nbr * qx.nbc)
    log(f"[bench] M={M} K={K} N={N} flagged blocks {n_fb} ({100 * f:.2f} %)")

    def step():
        fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta, out=qx)
        fq.fq_gemm(fq.FQ_OP_NT, qx, qw, out=y)

    # Warm-up: at least W steps and at least --warmup-seconds of back-to-back work, because the
    # GPU needs a few hundred milliseconds of load to leave its idle clock state.
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_w = time.perf_counter()
    while time.perf_counter() - t_w < args.warmup_seconds:
        for _ in range(20):
            step()
        torch.cuda.synchronize()

    # ---- timed region: exactly K steps, nothing else on the stream (a HIP event between the
    # kernels costs about 3 us each and would depress the whole-job number by 4 %)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps

    # ---- the same K steps once more, instrumented with HIP events on the launch stream, for
    # the per-kernel durations the roofline figures use
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        fq.fq_quantize(x, fq.FQ_CRIT_ABSMAX_GT, wl.theta, out=qx)
        ev[i][1].record()
        fq.fq_gemm(fq.FQ_OP_NT, qx, qw, out=y)
        ev[i][2].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step_instrumented = (t1 - t0) * 1e3 / args.steps
    ms_quant = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    ms_gemm = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))

    ops = 2.0 * M * N * K
    value = ops / (ms_step * 1e-3) / 1e12
    gemm_alg_ops = ops * (1.0 + f)          # the residual products are real MFMA work
    achieved = gemm_alg_ops / (ms_gemm * 1e-3) / 1e12
    quant_bytes = (3.0 + f) * M * K + 9.0 * qx.nbr * qx.nbc
    result = {
        "metric": "effective TOPS of quantize+fallback GEMM (% INT8 MFMA peak) vs bf16 GEMM, 1 GPU",
        "value": round(value, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": wl.name, "M": M, "K": K, "N": N, "block": 128,
                   "fallback_fraction": round(f, 5), "theta": wl.theta, "out_dtype": args.out_dtype,
                   "step": "fq_quantize(X) + fq_gemm(NT); W pre-quantized"},
        "pct_int8_peak": round(100.0 * value / INT8_PEAK_TOPS, 2),
        "ms_per_step_instrumented": round(ms_step_instrumented, 5),
        "ms_quantize": round(ms_quant, 5), "ms_gemm": round(ms_gemm, 5),
        "gemm_only_tops": round(ops / (ms_gemm * 1e-3) / 1e12, 2),
        "quantizer_gbs": round(quant_bytes / (ms_quant * 1e-3) / 1e9, 1),
        "roofline": {"bound": "mfma", "kernel": "fq::gemm_kernel",
                     "achieved": round(achieved, 2), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(achieved / INT8_PEAK_TOPS, 4),
                     "traffic": measured_gemm_traffic(wl.name)
                     if args.out_dtype == "bf16" else None,
                     "note": "INT8 ops: 2*M*N*K*(1+f) per launch / HIP-event time of fq_gemm, from "
                             "an instrumented repeat of the K timed steps (ms_per_step_instrumented)"},
    }

    # weight quantization (once per optimizer step in training), reported separately
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, out=qw)
    e0.record()
    for _ in range(10):
        fq.fq_quantize(w, fq.FQ_CRIT_NONE, 0.0, out=qw)
    e1.record()
    torch.cuda.synchronize()
    ms_wq = e0.elapsed_time(e1) / 10
    result["ms_quantize_weight"] = round(ms_wq, 5)
    result["tops_incl_weight_quant"] = round(ops / ((ms_step + ms_wq) * 1e-3) / 1e12, 2)

    if not args.no_bf16_baseline:
        yb = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        t_w = time.perf_counter()
        while time.perf_counter() - t_w < min(args.warmup_seconds, 1.0):
            for _ in range(10):
                torch.matmul(x, w.t(), out=yb)
            torch.cuda.synchronize()
        e0.record()
        for _ in range(50):
            torch.matmul(x, w.t(), out=yb)
        e1.record()
        torch.cuda.synchronize()
        ms_bf16 = e0.elapsed_time(e1) / 50
        result["bf16_gemm"] = {"impl": "torch.matmul (hipBLASLt)", "ms": round(ms_bf16, 5),
                               "tflops": round(ops / (ms_bf16 * 1e-3) / 1e12, 2),
                               "speedup_of_fq": round(ms_bf16 / ms_step, 3)}

    if not args.no_tolerance_variant:
        # fq_gemm_biased: the same product within a tolerance, half the dequantization work.  Not part
        # of `value` (the step times the exact kernel); reported beside it with its error.
        yv = torch.empty((M, N), dtype=out_dtype, device="cuda")
        ms_v = _time_loop(lambda: fq.fq_gemm_biased(fq.FQ_OP_NT, qx, qw, out=yv), min(args.warmup_seconds, 1.0), 100)
        exact32 = fq.fq_gemm(fq.FQ_OP_NT, qx, qw)
        var32 = fq.fq_gemm_biased(fq.FQ_OP_NT, qx, qw)
        err_v = ((var32.double() - exact32.double()).abs().max() / exact32.double().abs().max()).item()
        del exact32, var32, yv
        result["tolerance_variant"] = {
            "entry": "fq_gemm_biased", "ms_gemm": round(ms_v, 5),
            "mfma_tops": round(gemm_alg_ops / (ms_v * 1e-3) / 1e12, 2),
            "frac_of_int8_peak": round(gemm_alg_ops / (ms_v * 1e-3) / 1e12 / INT8_PEAK_TOPS, 4),
            "effective_tops_quant_plus_gemm": round(ops / ((ms_quant + ms_v) * 1e-3) / 1e12, 2),
            "max_abs_diff_over_max_abs_vs_fq_gemm_fp32": float(f"{err_v:.3e}"),
            "note": "fq_gemm is bit-identical to the CPU oracle; this variant is held to 1e-3"}

    if not args.no_mfma_ceiling:
        # what the INT8 matrix cores sustain with no memory traffic (power-limited; context for
        # roofline.frac, which stays relative to the published 5.0 POP/s)
        import subprocess
        tool = os.path.join(ROOT, "paper_2503_08040_amd", "mfma_ceiling")
        if os.path.exists(tool):
            torch.cuda.synchronize()
            r = subprocess.run([tool], capture_output=True, text=True, timeout=120)
            if r.returncode == 0:
                result["mfma_ceiling"] = json.loads(r.stdout.strip().splitlines()[-1])
    if not args.no_overhead_curve:
        log("[bench] config-5 overhead curve")
        result["overhead_curve_cfg5"] = overhead_curve()
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded sample")
        result["cpu_baseline"], window, oracle_out = cpu_baseline(wl)
        # the last timed step's output is still in y
        result["accuracy"] = accuracy(wl, window, oracle_out, y, x, w, qw)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
