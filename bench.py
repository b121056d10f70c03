#!/usr/bin/env python3
"""Benchmark of the partitioner's hot path on one MI355X.

One "step" = one full pass of the path over one synthetic data set already
resident in HBM: class split, quotas, similarity build of every class, and the
Algorithm-1 greedy of every class (gain sweeps, argmax, coverage updates),
through the C ABI entry point rcd_partition_dataset.

Prints ONE JSON line.  `value` = gain evaluations Algorithm 1 consumes per
second (sum over steps of the number of unassigned candidates, over the whole
job's wall time, similarity build included).  `roofline` covers the gain-sweep
kernel: algorithmic bytes (4 B per similarity entry of a live candidate column,
counted by the kernels themselves) over the kernel's time between HIP events
recorded around each of its launches in an extra, instrumented pass of the same
step.  `cpu_baseline` times the CPU oracle on a bounded sample on this host.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def describe(w, ds):
    return (f"{w.name}: {ds.L} classes x {w.n_c} samples, d={ds.X.shape[1]} {w.dtype}, K={len(ds.r)} "
            f"capacities {ds.r.tolist()}, Gaussian-mixture features, RBF sigma^2=d, seed {w.seed}")


def cpu_baseline(ds, budget_steps):
    """Oracle as it stands, one thread, on class 0 of the workload: its similarity
    matrix in full, then the first `budget_steps` greedy steps on it."""
    import oracle

    idx = np.flatnonzero(ds.labels == 0)
    n = len(idx)
    t0 = time.perf_counter()
    S0 = oracle.similarity(ds.X[idx], ds.sigma2)
    t_sim = time.perf_counter() - t0
    cap = oracle.quota(n, ds.r)
    # same proportions, cut to the window: the per-step work (|R_t| x n terms) is the real one
    win = np.floor(cap * (budget_steps / n)).astype(np.int64)
    win[-1] += budget_steps - win.sum()
    t0 = time.perf_counter()
    out = oracle.partition_class(S0, win)
    t_greedy = time.perf_counter() - t0
    steps = out["steps"]
    evals = sum(n - t for t in range(steps))
    # the graph-cut function on the same S: half the window (a marginal value walks a whole row here)
    gwin = win // 2
    t0 = time.perf_counter()
    gout = oracle.partition_class(S0, gwin, objective="gc")
    t_gc = time.perf_counter() - t0
    gc_evals = sum(n - t for t in range(gout["steps"]))
    # whole-job estimate: every class pays its similarity build and n(n+1)/2 gain evaluations
    job_evals = ds.L * n * (n + 1) / 2
    job_time = ds.L * t_sim + job_evals / (evals / t_greedy)
    return {
        "value": evals / t_greedy,
        "unit": "gain-evals/s",
        "cores": 1,
        "kind": "oracle",
        "sample": (f"class 0 of the workload (n={n}): the first {steps} greedy steps of the oracle on its own "
                   f"similarity matrix of that class ({evals} gain evaluations in {t_greedy:.2f} s); value = the rate "
                   f"measured in that window, nothing extrapolated (the matrix itself took {t_sim:.2f} s to build)"),
        "whole_job_evals_per_s_extrapolated": job_evals / job_time,
        "similarity_s_per_class": t_sim,
        "graph_cut_window_evals_per_s": gc_evals / t_gc if t_gc > 0 else None,
        "graph_cut_window": f"first {gout['steps']} steps of Algorithm 1 with the graph-cut function on the same S ({t_gc:.2f} s)",
        "host_cpus": os.cpu_count(),
    }


MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def extra_kernels(rcd, si, torch, only=""):
    """The matrix-core kernels and the HBM-clean sweep at the shape of one class of the large-class workload
    (50 000 x 2048 bf16, K = 8): the similarity build (default choice of tiles, and every tile), the bandwidth
    heuristic, the first rounds of a greedy run that recomputes S inside every sweep, and the same rounds
    streaming a stored 10 GB S.  Timed with events on the stream they run on.  `only` runs one of them (for a
    profiler): similarity, similarity_full, bandwidth, recompute, stored_sweep."""
    w = si.WORKLOADS["large"]
    n, d = w.n_c, w.d
    X = si.make_class(seed=w.seed, n=n, d=d, G=w.G, dtype="bf16")
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.bfloat16)
    res = {}
    reps = 3
    tiles = (n + 255) // 256
    want = lambda name: only in ("", name)

    def timed_similarity(mirror_env):
        S = torch.empty((n, n), dtype=torch.float32, device="cuda")
        ws = torch.empty(n * 4 + 256, dtype=torch.uint8, device="cuda")
        if mirror_env is not None:
            os.environ["RCD_SIM_MIRROR"] = mirror_env
        try:
            rcd.similarity(Xd, float(d), out=S, workspace=ws)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(reps):
                rcd.similarity(Xd, float(d), out=S, workspace=ws)
            e1.record()
            torch.cuda.synchronize()
        finally:
            if mirror_env is not None:
                del os.environ["RCD_SIM_MIRROR"]
        return e0.elapsed_time(e1) / reps

    if want("similarity"):
        ms = timed_similarity(None)
        executed = 2.0 * (tiles * (tiles + 1) // 2) * 256 * 256 * d
        tf = executed / (ms * 1e-3) / 1e12
        res["similarity_large_class"] = {
            "kernel": "sim::k_gram_rbf_fast<bf16, mirrored tiles> (+ row norms)", "shape": f"n={n} d={d} bf16 -> fp32 S",
            "ms": ms,
            "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                         "frac": tf / MFMA_PEAK_TFLOPS["bf16"],
                         "flops": "executed: 2 * 256 * 256 * d per tile, tiles on and above the diagonal only "
                                  "(each also stores its transpose)"},
            "nominal_2n2d_TFLOPs_per_s": 2.0 * n * n * d / (ms * 1e-3) / 1e12}
    if want("similarity_full"):
        # the same matrix by the full build (every tile computed, nothing mirrored): the matrix-core pipeline alone
        ms_full = timed_similarity("0")
        tf_full = 2.0 * tiles * tiles * 256 * 256 * d / (ms_full * 1e-3) / 1e12
        res.setdefault("similarity_large_class", {})["full_build"] = {
            "kernel": "sim::k_gram_rbf_fast<bf16, full> (RCD_SIM_MIRROR=0)", "ms": ms_full,
            "roofline": {"bound": "mfma", "achieved": tf_full, "peak": MFMA_PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                         "frac": tf_full / MFMA_PEAK_TFLOPS["bf16"], "flops": "executed: 2 * 256 * 256 * d per tile, every tile"}}
    if want("bandwidth"):
        # the paper's bandwidth heuristic on the same class: the same Gram tiles, on and above the diagonal only
        bws = torch.empty(rcd.load_library().rcd_bandwidth_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        sigma = rcd.bandwidth(Xd, workspace=bws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            rcd.bandwidth(Xd, workspace=bws)          # returns a host value: each call ends synchronised
        ms = 1e3 * (time.perf_counter() - t0) / reps
        flops = 2.0 * (tiles * (tiles + 1) // 2) * 256 * 256 * d
        tf = flops / (ms * 1e-3) / 1e12
        res["bandwidth_large_class"] = {
            "kernel": "sim::k_gram_rbf_fast<bf16, distance sum> (+ row norms, sum of tile sums, read-back)",
            "shape": f"n={n} d={d} bf16 -> sigma = mean pairwise L2 distance", "sigma": sigma, "ms": ms,
            "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                         "frac": tf / MFMA_PEAK_TFLOPS["bf16"],
                         "flops": "2 * 256 * 256 * d per tile, tiles on and above the diagonal"}}
        del bws
    if want("recompute"):
        # recompute mode: quotas cut to a 48-step window (same ratios), S never stored
        cap = np.array([2, 2, 4, 4, 6, 6, 8, 16], dtype=np.int64)
        rcd.profile(True)
        rcd.partition_class(X=Xd, cap=cap, sigma2=float(d))
        prof = rcd.profile_read()
        st = rcd.last_stats()
        rcd.profile(False)
        flops = 2.0 * st["entries_streamed"] * d
        tf = flops / (prof["sweep_ms"] * 1e-3) / 1e12 if prof["sweep_ms"] > 0 else 0.0
        res["recompute_sweep_large_class"] = {
            "kernel": "rcd_k_round_rc_fast<bf16> (S tiles rebuilt by MFMA inside the gain sweep)",
            "shape": f"n={n} d={d} bf16, K=8, first {st['steps']} greedy steps, {st['sweeps']} sweeps",
            "sweep_ms_total": prof["sweep_ms"], "steps_ms_total": prof["steps_ms"], "apply_ms_total": prof["apply_ms"],
            "useful_evals_per_s": st["useful_evals"] / ((prof["sweep_ms"] + prof["steps_ms"] + prof["apply_ms"]) * 1e-3),
            "roofline": {"bound": "mfma", "achieved": tf, "peak": MFMA_PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                         "frac": tf / MFMA_PEAK_TFLOPS["bf16"], "flops": "2 |R| n d per sweep"}}
    if want("stored_sweep"):
        res["stored_sweep_large_class"] = stored_sweep_large_class(rcd, torch, Xd, n, d)
    return res


def to_device(torch, ds):
    if ds.X.dtype == np.uint16:
        X = torch.from_numpy(ds.X.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        X = torch.from_numpy(ds.X).cuda()
    return X, torch.from_numpy(ds.labels).cuda()


def sweep_roofline(prof, pstats, note=None, n_class=None):
    """Roofline object of rcd_k_sweep_rows from an instrumented pass (HIP events around every launch)."""
    sweep_bytes = 4.0 * pstats["entries_streamed"]
    achieved = sweep_bytes / (prof["sweep_ms"] * 1e-3) / 1e9 if prof["sweep_ms"] > 0 else 0.0
    r = {"kernel": "rcd_k_sweep_rows (gain sweep of all stale blocks, stored similarity)", "bound": "hbm",
         "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
         "launches": prof["rounds"], "avg_launch_us": 1e3 * prof["sweep_ms"] / max(prof["rounds"], 1),
         "bytes_per_launch": sweep_bytes / max(prof["rounds"], 1), "sweeps_with_work": pstats["sweeps"]}
    if n_class:
        # sum over sweeps of (blocks x candidates) over sum of candidates: blocks evaluated per streamed entry
        r["avg_blocks_per_sweep"] = pstats["computed_evals"] * n_class / max(pstats["entries_streamed"], 1)
    if note:
        r["note"] = note
    return r


def one_config(rcd, si, torch, name, steps, warmup):
    """Partition wall time of one of the other workloads: by sweeps over a stored S (the route whose kernel the
    roofline covers) and by RCD_MODE_AUTO (what the library takes when left to choose), same protocol as the
    headline: inputs in HBM, `warmup` untimed passes, `steps` timed ones between synchronisations."""
    w = si.WORKLOADS[name]
    ds = si.make_dataset(w)
    X, labels = to_device(torch, ds)
    N, K = ds.X.shape[0], len(ds.r)
    counts = np.bincount(ds.labels, minlength=ds.L)
    _, full = rcd.dataset_workspace_bytes(N, ds.L, int(counts.max()), K, rcd.MODE_STORED)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")
    out = {"workload": describe(w, ds)}
    for label, mode in (("sweep_route", rcd.MODE_STORED), ("auto_route", rcd.MODE_AUTO)):
        for _ in range(warmup):
            rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, mode, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, mode, ws)
        torch.cuda.synchronize()
        sec = (time.perf_counter() - t0) / max(steps, 1)
        st = rcd.last_stats()
        out[label] = {"route": "RCD_MODE_STORED (one gain sweep per round)" if mode == rcd.MODE_STORED
                      else "RCD_MODE_AUTO (-> incremental gains: S fits the workspace)",
                      "partition_wall_time_ms": 1e3 * sec, "useful_evals_per_s": st["useful_evals"] / sec,
                      "greedy_steps": st["steps"], "sweeps": st["sweeps"], "kernel_launches": st["launches"],
                      "similarity_entries_read": st["entries_streamed"], "computed_evals": st["computed_evals"]}
    # the other two routes, one timed pass each after one warm-up: S rebuilt inside every sweep (nothing stored),
    # and Algorithm 1 with the graph-cut function of Section 4 on the stored S
    for label, kwargs, route in (("recompute_route", dict(mode=rcd.MODE_RECOMPUTE), "RCD_MODE_RECOMPUTE (S tiles rebuilt by the matrix cores inside every gain sweep)"),
                                 ("graph_cut_route", dict(mode=rcd.MODE_STORED, graph_cut=True), "rcd_partition_dataset_graph_cut (stored S)")):
        rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, workspace=ws, **kwargs)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, workspace=ws, **kwargs)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t0
        st = rcd.last_stats()
        out[label] = {"route": route, "partition_wall_time_ms": 1e3 * sec, "greedy_steps": st["steps"],
                      "useful_evals_per_s": st["useful_evals"] / sec, "runs_timed": 1}
    # instrumented pass of the sweep route: the sweep kernel at this workload's K
    rcd.profile(True)
    rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, rcd.MODE_STORED, ws)
    torch.cuda.synchronize()
    prof = rcd.profile_read()
    pst = rcd.last_stats()
    rcd.profile(False)
    total_S = float(np.sum(counts.astype(np.float64) ** 2) * 4)
    note = (f"K={K}: {pst['computed_evals'] / max(pst['useful_evals'], 1):.2f} gain evaluations computed per one consumed; "
            f"all classes' S together {total_S / 1e6:.0f} MB"
            + (" (fits the 256 MB Infinity Cache: not an HBM-clean figure)" if total_S < 256e6 else ""))
    out["sweep_kernel"] = sweep_roofline(prof, pst, note, n_class=w.n_c)
    out["time_split_ms"] = {"similarity": prof["similarity_ms"], "sweep": prof["sweep_ms"], "steps": prof["steps_ms"]}
    return out


def stored_sweep_large_class(rcd, torch, Xd, n, d):
    """The stored-S sweep kernel where no cache can help: one class of the large workload, S = 10 GB stored, K = 8,
    the first 48 greedy steps (quotas cut to a window, same ratios): every sweep streams the whole matrix."""
    cap = np.array([2, 2, 4, 4, 6, 6, 8, 16], dtype=np.int64)
    S = rcd.similarity(Xd, float(d))
    ws = torch.empty(rcd.class_workspace_bytes(n, len(cap), rcd.MODE_STORED), dtype=torch.uint8, device="cuda")
    rcd.partition_class(S=S, cap=cap, workspace=ws)          # warm-up
    rcd.profile(True)
    rcd.partition_class(S=S, cap=cap, workspace=ws)
    prof = rcd.profile_read()
    st = rcd.last_stats()
    rcd.profile(False)
    r = sweep_roofline(prof, st, "one 10 GB class: 40x the Infinity Cache, every byte from HBM", n_class=n)
    traffic_file = os.path.join(ROOT, "profiles", "sweep_traffic.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as fh:
            r["traffic"] = json.load(fh).get("large_class_hbm_bytes_per_launch")
    return {"shape": f"n={n}, S stored (fp32, {n * n * 4 / 1e9:.0f} GB), K=8, first {st['steps']} greedy steps, "
                     f"{st['sweeps']} sweeps", "sweep_ms_total": prof["sweep_ms"], "steps_ms_total": prof["steps_ms"],
            "roofline": r}


def large_workload(rcd, si, torch):
    """The whole large-class workload (20 classes x 50 000 samples, d = 2048 bf16, K = 8) by the
    incremental route with every class's similarity stored (200 GB of workspace): 1 000 000 greedy steps."""
    w = si.WORKLOADS["large"]
    try:
        ds = si.make_dataset(w)
        X = torch.from_numpy(ds.X.view(np.int16)).cuda().view(torch.bfloat16)
        labels = torch.from_numpy(ds.labels).cuda()
        _, full = rcd.dataset_workspace_bytes(len(ds.labels), ds.L, w.n_c, len(ds.r), rcd.MODE_INCREMENTAL)
        free, _ = torch.cuda.mem_get_info()
        if full > free * 0.95:
            return {"skipped": f"needs {full / 1e9:.0f} GB of workspace, {free / 1e9:.0f} GB free"}
        ws = torch.empty(full, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, rcd.MODE_INCREMENTAL, ws)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t0
        st = rcd.last_stats()
        out = {"workload": describe(w, ds), "route": "RCD_MODE_INCREMENTAL, every class's S stored",
               "partition_wall_time_s": sec, "greedy_steps": st["steps"],
               "useful_evals_per_s": st["useful_evals"] / sec, "similarity_entries_read": st["entries_streamed"],
               "workspace_GB": full / 1e9, "runs_timed": 1}
        # the same workload with the graph-cut function (one row of S per step, no update lists)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, workspace=ws, graph_cut=True)
        torch.cuda.synchronize()
        gsec = time.perf_counter() - t0
        gst = rcd.last_stats()
        out["graph_cut"] = {"route": "rcd_partition_dataset_graph_cut, every class's S stored",
                            "partition_wall_time_s": gsec, "greedy_steps": gst["steps"],
                            "useful_evals_per_s": gst["useful_evals"] / gsec, "runs_timed": 1}
        return out
    except Exception as e:       # e.g. not enough device or host memory on another box
        return {"skipped": repr(e)}


def whole_set_greedmax(rcd, torch, ds, X, class_wise_ms):
    """The same features as ONE class (no class split): the whole-set greedy that Section 3 compares the
    class-wise scheme with (pairwise work n^2 against n^2 / L), by the incremental route on the same kernels."""
    try:
        N, K = ds.X.shape[0], len(ds.r)
        labels0 = torch.zeros(N, dtype=torch.int32, device="cuda")
        _, full = rcd.dataset_workspace_bytes(N, 1, N, K, rcd.MODE_INCREMENTAL)
        free, _ = torch.cuda.mem_get_info()
        if full > free * 0.95:
            return {"skipped": f"needs {full / 1e9:.0f} GB of workspace, {free / 1e9:.0f} GB free"}
        ws = torch.empty(full, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rcd.partition_dataset(X, labels0, 1, ds.r, ds.sigma2, rcd.MODE_INCREMENTAL, ws)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t0
        st = rcd.last_stats()
        return {"workload": f"the bench workload's {N} samples as one class, K={K}", "route": "RCD_MODE_INCREMENTAL",
                "partition_wall_time_s": sec, "greedy_steps": st["steps"], "useful_evals_per_s": st["useful_evals"] / sec,
                "similarity_entries_read": st["entries_streamed"], "workspace_GB": full / 1e9, "runs_timed": 1,
                "class_wise_same_route_ms": class_wise_ms,
                "whole_set_over_class_wise_time": sec / (class_wise_ms * 1e-3)}
    except Exception as e:
        return {"skipped": repr(e)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cifar10")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the large-class similarity / recompute-sweep lines")
    ap.add_argument("--no-large", action="store_true", help="skip the whole large-class workload (200 GB of workspace)")
    ap.add_argument("--no-per-config", action="store_true", help="skip the wall times of the other workloads")
    ap.add_argument("--only", default="", choices=["", "large_workload", "similarity", "similarity_full", "bandwidth", "recompute",
                                                   "stored_sweep"],
                    help="run only this kernel of the large-class shape (50 000 x 2048 bf16), for a profiler")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy (known traffic) so that rocprofv3 byte counters can be scaled")
    ap.add_argument("--scale", default="", help="L,n_c,d override for quick runs (not a valid bench line)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2211_00839_amd as rcd
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: there is no CPU path", file=sys.stderr)
        sys.exit(2)
    rcd.load_library()
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "4 device copies of 1 GiB: each reads 2^30 B and writes 2^30 B"}))
        return

    if args.only == "large_workload":
        print(json.dumps({"large_workload_incremental": large_workload(rcd, si, torch)}))
        return
    if args.only:
        print(json.dumps(extra_kernels(rcd, si, torch, only=args.only)))
        return

    w = si.WORKLOADS[args.workload]
    kw = {}
    if args.scale:
        L, n_c, d = (int(x) for x in args.scale.split(","))
        kw = dict(L=L, n_c=n_c, d=d)
    ds = si.make_dataset(w, **kw)
    N, d = ds.X.shape
    K = len(ds.r)
    if ds.X.dtype == np.uint16:
        X = torch.from_numpy(ds.X.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        X = torch.from_numpy(ds.X).cuda()
    labels = torch.from_numpy(ds.labels).cuda()
    counts = np.bincount(ds.labels, minlength=ds.L)
    _, full = rcd.dataset_workspace_bytes(N, ds.L, int(counts.max()), K, rcd.MODE_STORED)
    ws = torch.empty(full, dtype=torch.uint8, device="cuda")

    def step():
        return rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, rcd.MODE_STORED, ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        assign, order, obj = step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stats = rcd.last_stats()
    ms_per_step = 1e3 * elapsed / max(args.steps, 1)
    value = stats["useful_evals"] / (ms_per_step * 1e-3)

    # instrumented pass of the same step: HIP events around every launch of a round
    rcd.profile(True)
    t1 = time.perf_counter()
    step()
    torch.cuda.synchronize()
    prof_ms = 1e3 * (time.perf_counter() - t1)
    prof = rcd.profile_read()
    pstats = rcd.last_stats()
    rcd.profile(False)
    roofline = sweep_roofline(prof, pstats, n_class=int(counts.max()))
    traffic_file = os.path.join(ROOT, "profiles", "sweep_traffic.json")
    if os.path.exists(traffic_file) and not args.scale and args.workload == "cifar10":
        with open(traffic_file) as fh:
            roofline["traffic"] = json.load(fh).get("hbm_bytes_per_launch")

    # the same step by the incremental-gain route (same Algorithm 1, same answers: gains are moved by the
    # rows of S whose coverage changed instead of rebuilt by sweeps)
    def step_inc():
        return rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, rcd.MODE_INCREMENTAL, ws)

    step_inc()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        a_inc, o_inc, f_inc = step_inc()
    torch.cuda.synchronize()
    inc_ms = 1e3 * (time.perf_counter() - t2) / max(args.steps, 1)
    istats = rcd.last_stats()
    incremental = {
        "route": "RCD_MODE_INCREMENTAL on the same workload, same timing protocol",
        "ms_per_step": inc_ms,
        "value": istats["useful_evals"] / (inc_ms * 1e-3),
        "unit": "gain-evals/s",
        "similarity_entries_read": istats["entries_streamed"],
        "similarity_entries_read_by_sweeps": stats["entries_streamed"],
        "kernel_launches": istats["launches"],
        "same_assignment_as_sweep_route": bool(torch.equal(a_inc, assign)),
    }

    # Algorithm 1 with the graph-cut function of Section 4 on the same workload (stored S, same protocol)
    def step_gc():
        return rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, workspace=ws, graph_cut=True)

    step_gc()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    for _ in range(args.steps):
        step_gc()
    torch.cuda.synchronize()
    gc_ms = 1e3 * (time.perf_counter() - t3) / max(args.steps, 1)
    gstats = rcd.last_stats()
    n_max = int(counts.max())
    graph_cut = {
        "route": "rcd_partition_dataset_graph_cut on the same workload, same timing protocol",
        "ms_per_step": gc_ms,
        "value": gstats["useful_evals"] / (gc_ms * 1e-3),
        "unit": "gain-evals/s",
        "greedy_steps": gstats["steps"],
        "kernel_launches": gstats["launches"],
        # a step reads the block's marginal values (8 B each), one row of S (4 B) and rewrites the values (16 B)
        "bytes_per_greedy_step": 28 * n_max,
        "us_per_greedy_step_in_loop": 10e-3 * gstats["step_ticks"] / max(gstats["steps"], 1) ,
        "bound": "latency of one workgroup's step (scan, two barriers, one row): classes run side by side, one compute unit each",
    }

    # the same workload with nothing stored: S tiles rebuilt by the matrix cores inside every gain sweep (one timed pass)
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    rcd.partition_dataset(X, labels, ds.L, ds.r, ds.sigma2, rcd.MODE_RECOMPUTE, ws)
    torch.cuda.synchronize()
    rc_ms = 1e3 * (time.perf_counter() - t4)
    rstats = rcd.last_stats()
    recompute = {"route": "RCD_MODE_RECOMPUTE on the same workload, one timed pass", "ms_per_step": rc_ms,
                 "value": rstats["useful_evals"] / (rc_ms * 1e-3), "unit": "gain-evals/s", "greedy_steps": rstats["steps"],
                 "kernel_launches": rstats["launches"], "runs_timed": 1}

    out = {
        "metric": "marginal-gain evals/sec (gain evaluations Algorithm 1 consumes / whole-job wall time)",
        "value": value,
        "unit": "gain-evals/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if ds.X.dtype == np.float32 else "bf16",
        "data": "synthetic",
        "config": {"workload": describe(w, ds), "mode": "stored S, all classes advanced together",
                   "scaled_down": bool(args.scale)},
        "partition_wall_time_s": ms_per_step * 1e-3,
        "useful_evals_per_step": stats["useful_evals"],
        "computed_evals_per_step": stats["computed_evals"],
        "greedy_steps": stats["steps"],
        "sweeps": stats["sweeps"],
        "kernel_launches": stats["launches"],
        "time_split_ms": {"similarity": prof["similarity_ms"], "sweep": prof["sweep_ms"], "steps": prof["steps_ms"],
                          "apply": prof["apply_ms"], "instrumented_step_total": prof_ms},
        "roofline": roofline,
        "incremental_route": incremental,
        "graph_cut_route": graph_cut,
        "recompute_route": recompute,
    }
    if not args.scale and not args.no_per_config:
        # the other workloads of the configuration list (the large one is under `extra`)
        out["per_config"] = {name: one_config(rcd, si, torch, name, args.steps, args.warmup)
                             for name in ("tiny", "hetero8", "cifar100") if name != args.workload}
    if not args.scale and not args.no_extra:
        del ws
        out["extra"] = extra_kernels(rcd, si, torch)
        out["extra"]["whole_set_greedmax"] = whole_set_greedmax(rcd, torch, ds, X, inc_ms)
        if not args.no_large:
            out["extra"]["large_workload_incremental"] = large_workload(rcd, si, torch)
    if not args.no_cpu_baseline:
        n0 = int(counts[0])
        out["cpu_baseline"] = cpu_baseline(ds, budget_steps=min(320, n0))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
