#!/usr/bin/env python3
"""Benchmark of the LCN-Sinkhorn hot path on one MI355X.

One step = one pass of the whole path on one synthetic problem already in HBM:
lcn_build (landmarks, LSH buckets, bucket sort, Nystrom factors, sparse
correction) + sinkhorn_run(iters) + transport_cost.  The headline value is
Sinkhorn iterations per second inside sinkhorn_run (HIP events on the
library's stream); build time and the whole step are reported beside it.

Prints ONE JSON line.  roofline.achieved = algorithmic bytes of one
half-iteration launch (every factor entry and every sparse value once) divided
by the average duration of such a launch, from HIP events around sinkhorn_run;
roofline.traffic = HBM bytes per launch from the hardware counters: read, at
run time, from the counter table of the rocprofv3 summary under profiles/ that
covers the workload (null if that file has no such row).

The default run (configuration 3, the metric's) also carries a short record
"c5" for configuration 5 (n = m = 200 000, where the sweep is bound by HBM and
not by launch latency) and times the oracle twice: on all host cores and on one.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP64_VECTOR_PEAK_TFLOPS = 78.6   # MI355X, published


def make_problem(config: int, lam_factor: float = 0.05):
    import workloads
    if config == 2 and lam_factor != 0.05:
        return (workloads.config2(lam_factor=lam_factor),
                "C2 n=m=10000 d=64 sq-Euclid lambda=%g*median l=128 b=64x2 it=100" % lam_factor)
    if config == 1:
        return workloads.config1(), "C1 n=m=1024 d=16 sq-Euclid l=64 b=16x1 it=50"
    if config == 2:
        return workloads.config2(), "C2 n=m=10000 d=64 sq-Euclid l=128 b=64x2 it=100"
    if config == 3:
        return workloads.config3(), "C3 n=m=20000 d=300 cosine lambda=0.05 l=256 b=128x3 it=200"
    if config == 5:
        return workloads.config5(), "C5 n=m=200000 d=300 bf16-in cosine lambda=0.05 l=512 b=1024x3 it=200"
    raise SystemExit("unknown --config %d" % config)


def _omp_threads(n=None):
    """Thread count of the OpenMP runtime the oracle runs on; sets it first if n is given."""
    import ctypes
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        if n is not None:
            gomp.omp_set_num_threads(int(n))
        return int(gomp.omp_get_max_threads())
    except OSError:
        return int(os.environ.get("OMP_NUM_THREADS", "0")) or os.cpu_count()


def counter_traffic(config: int):
    """HBM bytes per pass_kernel launch from the counter table of the profile summary of this
    configuration (scaled read MB + scaled write MB of the fused update sweep), or None."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "lcn_sinkhorn_c%d_*.md" % config))):
        for line in open(path):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 6 and re.match(r"`pass_kernel<.*true>`", cells[1]):
                try:
                    return (float(cells[5]) + float(cells[6])) * 1e6
                except ValueError:
                    pass
    return None


def _cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(p, sample_iters: int, one_thread_iters: int = 0):
    """The oracle as it stands on the host cores: full build of the same
    problem, then a few iterations; then (one_thread_iters > 0) a shorter run on
    one thread."""
    import oracle
    threads = _omp_threads()
    t0 = time.perf_counter()
    B = oracle.build_problem(p.X, p.Y, p.cost, p.lam, "lcn", p.num_landmarks, p.landmark_seed, p.kmeans_iters,
                             p.ridge, 0, p.num_buckets, p.num_rounds, p.lsh_seed, p.projections,
                             landmark_init=p.landmark_init, landmark_iters=p.landmark_iters, branching=p.branching)
    t1 = time.perf_counter()
    st = oracle.sinkhorn(B.op, p.a, p.b, sample_iters)
    t2 = time.perf_counter()
    _, _, dist, resid = oracle.marginals(B.op, p.a, p.b, p.lam, st)
    out = {
        "value": sample_iters / (t2 - t1), "unit": "iterations/s", "cores": threads, "kind": "oracle",
        "sample": "full oracle build of the same problem (%.1f s) then %d Sinkhorn iterations (%.2f s)"
                  % (t1 - t0, sample_iters, t2 - t1),
        "build_ms": 1e3 * (t1 - t0), "cpu_model": _cpu_model(), "host_cpus": os.cpu_count(),
    }
    if one_thread_iters > 0:
        _omp_threads(1)
        t3 = time.perf_counter()
        oracle.sinkhorn(B.op, p.a, p.b, one_thread_iters)
        t4 = time.perf_counter()
        _omp_threads(threads)
        out["one_thread"] = {"value": one_thread_iters / (t4 - t3), "unit": "iterations/s", "cores": 1,
                             "sample": "%d Sinkhorn iterations of the same problem on one thread (%.2f s)"
                                       % (one_thread_iters, t4 - t3)}
    return out, (st, dist, resid)


def timed_run(config: int, mode_name: str, steps: int, warmup: int):
    """A short run of the whole path on another configuration (same step as the main loop:
    lcn_build + sinkhorn_run + transport_cost, inputs resident, workspace reused): its iterations/s,
    build time and the roofline of its half-iteration kernel."""
    import numpy as np
    import torch

    import paper_2107_06876_amd as lcn

    p, wl = make_problem(config)
    dev = "cuda:0"
    dt = torch.bfloat16 if p.bf16_inputs else torch.float32
    X = torch.from_numpy(p.X).to(dev).to(dt)
    Y = torch.from_numpy(p.Y).to(dev).to(dt)
    a = torch.from_numpy(p.a).to(dev)
    b = torch.from_numpy(p.b).to(dev)
    mode = {"lcn": lcn.MODE_LCN, "sparse": lcn.MODE_SPARSE, "nystrom": lcn.MODE_NYSTROM, "dense": lcn.MODE_DENSE}[mode_name]
    lm = dict(num_landmarks=p.num_landmarks, kmeans_iters=p.kmeans_iters, seed=p.landmark_seed, ridge=p.ridge)
    lsh = dict(hash=lcn.HASH_KMEANS, num_buckets=p.num_buckets, num_rounds=p.num_rounds,
               kmeans_iters=p.kmeans_iters, seed=p.lsh_seed)
    h = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, mode, landmarks=lm, lsh=lsh)
    ws = h.workspace
    info = lcn.lcn_get_info(h)
    lcn.lcn_destroy(h)
    build_ms, run_ms, launches, dist = [], [], 0, None
    t0 = None
    for it in range(warmup + steps):
        if it == warmup:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
        tb = time.perf_counter()
        hh = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, mode, landmarks=lm, lsh=lsh, workspace=ws)
        te = time.perf_counter()
        lcn.sinkhorn_run(hh, p.iters)
        ms, launches = lcn.lcn_last_run_timing(hh)
        dist = lcn.transport_cost(hh)
        lcn.lcn_destroy(hh)
        if it >= warmup:
            build_ms.append(1e3 * (te - tb))
            run_ms.append(ms)
    torch.cuda.synchronize()
    ms_per_step = 1e3 * (time.perf_counter() - t0) / steps
    run_mean = float(np.mean(run_ms))
    bytes_launch = (4.0 * (p.n * info.l + info.l * p.m) + 8.0 * info.nnz_unique) / 2.0
    launch_us = run_mean * 1e3 / max(launches, 1)
    achieved = bytes_launch / (launch_us * 1e-6) / 1e9
    del X, Y, ws
    torch.cuda.empty_cache()
    return {"workload": wl, "steps": steps, "warmup": warmup, "value": p.iters / (run_mean * 1e-3),
            "unit": "iterations/s", "ms_per_step": ms_per_step, "build_ms": float(np.mean(build_ms)),
            "sinkhorn_ms": run_mean, "distance": dist, "nnz_unique": info.nnz_unique,
            "roofline": {"bound": "hbm", "kernel": "pass_kernel (one half-iteration)", "achieved": achieved,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                         "traffic": counter_traffic(config), "bytes_per_launch": bytes_launch,
                         "launch_us": launch_us}}


def plan_measures(h_approx, h_exact, n):
    """Pearson correlation of all plan entries and overlap (IoU) of the 0.1 % largest ones between an
    approximate plan and the dense one (the other two columns of the paper's accuracy table, Sec. 8)."""
    import torch

    import paper_2107_06876_amd as lcn
    Pa = lcn.lcn_plan_rows(h_approx, 0, n).flatten()
    Pe = lcn.lcn_plan_rows(h_exact, 0, n).flatten()
    x, y = Pa.double(), Pe.double()
    xm, ym = x.mean(), y.mean()
    pcc = float(((x - xm) * (y - ym)).sum() / torch.sqrt(((x - xm) ** 2).sum() * ((y - ym) ** 2).sum()))
    k = max(Pa.numel() // 1000, 1)
    ta = torch.topk(Pa, k).indices
    te = torch.topk(Pe, k).indices
    inter = int(torch.isin(ta, te).sum())
    return pcc, inter / (2 * k - inter)


def accuracy_table():
    """Relative error of the Sinkhorn distance, PCC and IoU of LCN-Sinkhorn against dense Sinkhorn
    (Table 1's three columns) on configuration 1, on configuration 2 at the largest-but-one lambda
    where its LCN path stays positive (0.5 x median; at the configuration's own 0.05 x median both sides
    report non-positive sums), and on the paper's own synthetic workload (uniform in the d-ball,
    d = 16, n = 10^4, lambda = 0.05: Table 1 prints 0.435 / 0.328 / 0.079 for LCN).  Outside the timed
    region; everything through the library."""
    import torch

    import paper_2107_06876_amd as lcn
    import workloads
    out = {}
    dev = "cuda:0"
    for name, p in (("c1", workloads.config1()), ("c2_lambda_0.5_median", workloads.config2(lam_factor=0.5)),
                    ("dball", workloads.dball())):
        X, Y = torch.from_numpy(p.X).to(dev), torch.from_numpy(p.Y).to(dev)
        a, b = torch.from_numpy(p.a).to(dev), torch.from_numpy(p.b).to(dev)
        lm = dict(num_landmarks=p.num_landmarks, kmeans_iters=p.kmeans_iters, seed=p.landmark_seed, ridge=p.ridge)
        lsh = dict(hash=lcn.HASH_KMEANS, num_buckets=p.num_buckets, num_rounds=p.num_rounds,
                   kmeans_iters=p.kmeans_iters, seed=p.lsh_seed)
        try:
            hd = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, lcn.MODE_DENSE)
            lcn.sinkhorn_run(hd, p.iters)
            hl = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, lcn.MODE_LCN, landmarks=lm, lsh=lsh)
            lcn.sinkhorn_run(hl, p.iters)
            d_d, d_l = lcn.transport_cost(hd), lcn.transport_cost(hl)
            pcc, iou = plan_measures(hl, hd, p.n)
            out[name] = {"cost_rel_err_vs_dense": abs(d_l - d_d) / abs(d_d), "pcc": pcc, "iou_top_0.1pct": iou,
                         "distance_lcn": d_l, "distance_dense": d_d}
            lcn.lcn_destroy(hl)
            lcn.lcn_destroy(hd)
            del hl, hd
        except lcn.LcnError as e:
            out[name] = {"note": str(e)}
        torch.cuda.empty_cache()
    return out


def bench_batched(args):
    """Config 4: 1024 small pairs with deletion rows/columns, one launch."""
    import numpy as np
    import torch

    import paper_2107_06876_amd as lcn
    import workloads

    B = workloads.config4()
    dev = "cuda:0"
    X = torch.from_numpy(B.X).to(dev)
    Y = torch.from_numpy(B.Y).to(dev)
    dx = torch.from_numpy(B.del_x).to(dev)
    dy = torch.from_numpy(B.del_y).to(dev)
    lm = dict(num_landmarks=B.num_landmarks, kmeans_iters=B.kmeans_iters, seed=B.landmark_seed, ridge=B.ridge)
    lsh = dict(num_buckets=B.num_buckets, num_rounds=1, kmeans_iters=B.kmeans_iters, seed=B.lsh_seed)
    ws = None

    def step():
        nonlocal ws
        t0 = time.perf_counter()
        h = lcn.lcn_build_batched(X, Y, B.x_off, B.y_off, B.lam, B.cost, lcn.MODE_LCN, dx, dy, landmarks=lm, lsh=lsh,
                                  workspace=ws)
        ws = h.workspace
        t1 = time.perf_counter()
        lcn.sinkhorn_run(h, B.iters)
        ms, _ = lcn.lcn_last_run_timing(h)
        dist, resid = lcn.lcn_batched_results(h)
        lcn.lcn_destroy(h)
        return 1e3 * (t1 - t0), ms, dist

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    bms, rms = [], []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        b, r, dist = step()
        bms.append(b)
        rms.append(r)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run_mean = float(np.mean(rms))
    P = B.num_problems
    flops = 4.0 * float(np.sum(np.diff(B.x_off) * np.diff(B.y_off))) * B.iters
    out = {
        "metric": "batched LCN-Sinkhorn (1024 pairs): aggregate Sinkhorn iterations/s", "value": P * B.iters / (run_mean * 1e-3),
        "unit": "iterations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * (t1 - t0) / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 storage, f64 accumulate", "data": "synthetic",
        "config": {"workload": "C4 1024 pairs n,m in [16,64] d=32 Euclid + deletion cost 1, l=8 b=4 it=50", "mode": "lcn"},
        "build_ms": float(np.mean(bms)), "sinkhorn_ms": run_mean, "pairs_per_s": P / (run_mean * 1e-3),
        "mean_distance": float(np.mean(dist)),
        "roofline": {"bound": "alu", "kernel": "batched_run_kernel", "achieved": flops / (run_mean * 1e-3) / 1e12,
                     "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": flops / (run_mean * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS, "traffic": None,
                     "note": "4 n m fp64 flops per pair and iteration (two products with the n x m tile); one "
                             "wavefront per pair in registers: bound by the latency of a single instruction "
                             "stream, neither HBM nor MFMA"},
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-accuracy", action="store_true")
    ap.add_argument("--no-c5", action="store_true",
                    help="leave out the short record for configuration 5 that the default run carries")
    ap.add_argument("--no-peaks", action="store_true",
                    help="leave out the measured ceilings of the part (copy and read bandwidth, matrix-instruction "
                         "rates, empty-launch cost) that the line otherwise carries under measured_peaks")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a 256 MiB device-to-device copy so that rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                         "can be scaled by what the same counter reads for a copy of known size")
    ap.add_argument("--cpu-iters", type=int, default=1000,
                    help="Sinkhorn iterations of the oracle sample (with its build: about 10 s of CPU work at C3)")
    ap.add_argument("--mode", default="lcn", choices=["lcn", "sparse", "nystrom", "dense"])
    ap.add_argument("--landmarks", default="kmeans", choices=["kmeans", "kmeans++"],
                    help="kmeans: the configuration's k-means landmarks; kmeans++: landmarks sampled by "
                         "k-means++ seeding, no Lloyd iterations")
    ap.add_argument("--lam-factor", type=float, default=0.05,
                    help="configuration 2 only: lambda as a multiple of the median cost (at the configuration's "
                         "own 0.05 the Nystrom part goes negative and the run ends with that status; 0.5 runs)")
    ap.add_argument("--branching", default="",
                    help="hierarchical k-means hashing: comma-separated factors whose product is the "
                         "configuration's bucket count, e.g. 32,32 (default: flat k-means)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
                         "--gpus %d is not supported" % args.gpus)
    if args.config == 4:
        return bench_batched(args)

    import numpy as np
    import torch

    import paper_2107_06876_amd as lcn
    import workloads

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    p, wl = make_problem(args.config, args.lam_factor)
    dev = "cuda:0"
    dt = torch.bfloat16 if p.bf16_inputs else torch.float32
    X = torch.from_numpy(p.X).to(dev).to(dt)
    Y = torch.from_numpy(p.Y).to(dev).to(dt)
    a = torch.from_numpy(p.a).to(dev)
    b = torch.from_numpy(p.b).to(dev)
    mode = {"lcn": lcn.MODE_LCN, "sparse": lcn.MODE_SPARSE, "nystrom": lcn.MODE_NYSTROM, "dense": lcn.MODE_DENSE}[args.mode]
    lm = dict(num_landmarks=p.num_landmarks, kmeans_iters=p.kmeans_iters, seed=p.landmark_seed, ridge=p.ridge)
    if args.landmarks == "kmeans++":
        p.landmark_init, p.landmark_iters = "kmeans++", 0
        lm.update(init=lcn.INIT_KMEANSPP, kmeans_iters=0)
        wl += " landmarks=kmeans++ sampling"
    lsh = dict(hash=lcn.HASH_KMEANS, num_buckets=p.num_buckets, num_rounds=p.num_rounds,
               kmeans_iters=p.kmeans_iters, seed=p.lsh_seed)
    if args.branching:
        p.branching = tuple(int(x) for x in args.branching.split(","))
        lsh["branching"] = p.branching
        wl += " hierarchical k-means " + "x".join(str(x) for x in p.branching)
    lm = lm if args.mode in ("lcn", "nystrom") else None
    lsh = lsh if args.mode in ("lcn", "sparse") else None

    if args.config == 3 and args.mode == "lcn" and not args.no_c5:
        c5 = timed_run(5, "lcn", 3, 1)
    else:
        c5 = None

    # first build sizes the workspace; every later build reuses it (no allocation in the timed region)
    h = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, mode, landmarks=lm, lsh=lsh)
    ws = h.workspace
    info = lcn.lcn_get_info(h)
    nnz_stored, nnz_unique, l = info.nnz_stored, info.nnz_unique, info.l
    lcn.lcn_destroy(h)

    def step():
        t0 = time.perf_counter()
        hh = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, mode, landmarks=lm, lsh=lsh, workspace=ws)
        t1 = time.perf_counter()          # lcn_build returns after its work has finished
        lcn.sinkhorn_run(hh, p.iters)
        ms, launches = lcn.lcn_last_run_timing(hh)
        d = lcn.transport_cost(hh)
        return hh, 1e3 * (t1 - t0), ms, launches, d

    try:
        hh, *_ = step()
        lcn.lcn_destroy(hh)
    except lcn.LcnError as e:
        # a configuration on which the method itself fails (configuration 2 as specified: App. "Limitations")
        print(json.dumps({"metric": "LCN-Sinkhorn iterations/s", "value": None, "unit": "iterations/s", "n_gpus": 1,
                          "status": str(e), "config": {"workload": wl, "mode": args.mode}}))
        raise SystemExit(1)
    for _ in range(args.warmup):
        hh, *_ = step()
        lcn.lcn_destroy(hh)
    torch.cuda.synchronize()
    build_ms, run_ms, n_launch = [], [], 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        hh, bms, ms, launches, dist = step()
        build_ms.append(bms)
        run_ms.append(ms)
        n_launch = launches
        lcn.lcn_destroy(hh)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = 1e3 * (t1 - t0) / args.steps
    run_mean = float(np.mean(run_ms))
    its_per_s = p.iters / (run_mean * 1e-3)

    # roofline of the half-iteration kernel: algorithmic bytes per launch = half of
    # 4 (n l + l m) + 2 * 4 * nnz  (each factor entry once, each sparse value twice per iteration)
    bytes_iter = 4.0 * (p.n * l + l * p.m) + 8.0 * nnz_unique
    bytes_launch = bytes_iter / 2.0
    launch_us = run_mean * 1e3 / max(n_launch, 1)
    achieved = bytes_launch / (launch_us * 1e-6) / 1e9
    # HBM bytes per pass_kernel launch from the rocprofv3 counter runs (FETCH_SIZE scaled by 2.000 plus
    # WRITE_SIZE scaled by 1.000 against a 256 MiB device copy); see profiles/lcn_sinkhorn_c*.md
    traffic = counter_traffic(args.config) if args.mode == "lcn" else None
    out = {
        "metric": "LCN-Sinkhorn iterations/s (n=20k,d=300); build ms; % HBM peak; cost rel.err",
        "value": its_per_s, "unit": "iterations/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 storage, f64 accumulate", "data": "synthetic",
        "config": {"workload": wl, "mode": args.mode, "iters": p.iters, "nnz_unique": nnz_unique,
                   "nnz_stored": nnz_stored},
        "build_ms": float(np.mean(build_ms)), "sinkhorn_ms": run_mean, "distance": dist,
        "roofline": {"bound": "hbm", "kernel": "pass_kernel (one half-iteration)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "bytes_per_launch": bytes_launch, "launch_us": launch_us},
    }
    if c5 is not None:
        out["c5"] = c5
    if not args.no_peaks:
        # what this part reaches in place (lcn_calibrate): the published peaks stay the roofline's denominator
        try:
            buf = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
            out["measured_peaks"] = {
                "copy_GBs_read_plus_write": lcn.lcn_calibrate(lcn.CAL_COPY_GBS, buf),
                "read_GBs": lcn.lcn_calibrate(lcn.CAL_READ_GBS, buf),
                "mfma_bf16_32x32x16_TFLOPs": lcn.lcn_calibrate(lcn.CAL_MFMA_BF16_TFLOPS, buf),
                "mfma_f64_16x16x4_TFLOPs": lcn.lcn_calibrate(lcn.CAL_MFMA_F64_TFLOPS, buf),
                "empty_launch_us": lcn.lcn_calibrate(lcn.CAL_LAUNCH_US, buf),
                "published": {"hbm_GBs": HBM_PEAK_GBS, "mfma_bf16_TFLOPs": 2500.0, "mfma_f64_TFLOPs": 78.6}}
            del buf
        except Exception as e:  # noqa: BLE001
            out["measured_peaks"] = {"note": str(e)}
    if args.copy_calibration:
        src = torch.empty(64 << 20, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration_bytes_each_way"] = src.numel() * 4
    if args.config in (1, 2, 3) and args.mode == "lcn" and not args.no_accuracy:
        # accuracy of the approximation (Table 1's first column): the dense sibling on the GPU, outside the timed region
        try:
            hd = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, lcn.MODE_DENSE)
            lcn.sinkhorn_run(hd, p.iters)
            d_dense = lcn.transport_cost(hd)
            lcn.lcn_destroy(hd)
            del hd
            out["cost_rel_err_vs_dense"] = abs(dist - d_dense) / abs(d_dense)
            out["distance_dense"] = d_dense
        except lcn.LcnError as e:
            out["cost_rel_err_vs_dense"] = None
            out["accuracy_note"] = str(e)
    if args.config == 3 and args.mode == "lcn" and not args.no_accuracy:
        # The same comparison on the pre-aligned variant (Y rotated back, matched rows close, as after
        # the Procrustes step of the paper's embedding runs): there the dense distance is not a
        # near-cancellation of transport cost and entropy, and the relative error means something.
        pa = workloads.config3(prealigned=True, name="C3 prealigned")
        Ya = torch.from_numpy(pa.Y).to(dev)
        try:
            hl = lcn.lcn_build(X, Ya, a, b, pa.lam, pa.cost, mode, landmarks=lm, lsh=lsh)
            lcn.sinkhorn_run(hl, pa.iters)
            d_l = lcn.transport_cost(hl)
            lcn.lcn_destroy(hl)
            del hl
            hd = lcn.lcn_build(X, Ya, a, b, pa.lam, pa.cost, lcn.MODE_DENSE)
            lcn.sinkhorn_run(hd, pa.iters)
            d_d = lcn.transport_cost(hd)
            lcn.lcn_destroy(hd)
            del hd
            out["prealigned"] = {"distance_lcn": d_l, "distance_dense": d_d,
                                 "cost_rel_err_vs_dense": abs(d_l - d_d) / abs(d_d)}
        except lcn.LcnError as e:
            out["prealigned"] = {"note": str(e)}
    if args.config == 3 and args.mode == "lcn" and not args.no_accuracy:
        out["accuracy_table"] = accuracy_table()
    if args.mode in ("lcn", "nystrom") and not args.no_accuracy:
        # analytic derivatives (Prop. 1) of the converged state, outside the timed region
        hb = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, mode, landmarks=lm, lsh=lsh, workspace=ws)
        lcn.sinkhorn_run(hb, p.iters)
        nnz_b = int(lcn.lcn_get_csr(hb)[1].numel()) if args.mode == "lcn" else 0
        lcn.lcn_backward(hb, nnz_b)          # allocates its outputs; the second call is the timed one
        torch.cuda.synchronize()
        tb = time.perf_counter()
        lcn.lcn_backward(hb, nnz_b)
        out["backward_ms"] = 1e3 * (time.perf_counter() - tb)
        lcn.lcn_destroy(hb)
    if not args.no_cpu_baseline:
        base, (st, dist_o, resid_o) = cpu_baseline(p, args.cpu_iters, max(1, args.cpu_iters // 8))
        out["cpu_baseline"] = base
        # parity of a short GPU run against the same oracle run (outside the timed region)
        hh = lcn.lcn_build(X, Y, a, b, p.lam, p.cost, mode, landmarks=lm, lsh=lsh, workspace=ws)
        lcn.sinkhorn_run(hh, args.cpu_iters)
        lu, lv = lcn.lcn_get_scalings(hh)
        d5 = lcn.transport_cost(hh)
        out["parity_vs_oracle"] = {
            "iters": args.cpu_iters,
            "max_abs_log_u": float(np.max(np.abs(lu.cpu().numpy() - st.log_u))),
            "max_abs_log_v": float(np.max(np.abs(lv.cpu().numpy() - st.log_v))),
            "cost_rel": abs(d5 - dist_o) / abs(dist_o)}
        lcn.lcn_destroy(hh)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
