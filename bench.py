#!/usr/bin/env python3
"""Benchmark of the batched matrix exponential on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C5f64] [--no-others] [--no-cpu] [--no-extras]

A step is one expm() call over one synthetic batch that is already resident in HBM: norms,
selection of (m, s), polynomial evaluation, squarings and the store of the result.  Prints one
JSON line: the headline workload (by default the largest one, 4 matrices of order 4096 in fp64) plus, under
"per_config", the same figures for all workloads.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"hbm": 8000.0, "mfma_f32": 157.3, "mfma_f64": 78.6}  # GB/s, TFLOP/s (MI355X published)
DEFAULT_STEPS = {"F1": 1000, "C1": 1000, "C2": 1000, "C3": 100, "C4": 60, "C5f64": 20, "C5f32": 20, "L1": 100}
DEFAULT_WARMUP = {"F1": 500, "C1": 500, "C2": 500, "C3": 20, "C4": 15, "C5f64": 3, "C5f32": 3, "L1": 10}


def source_sha1():
    import glob
    import hashlib
    h = hashlib.sha1()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2512_20777_amd", "csrc", "*"))):
        h.update(open(f, "rb").read())
    return h.hexdigest()


def recorded_traffic(workload, kernel_prefix):
    """HBM bytes per dispatch of the kernel from the committed counter summary (profiles/hbm_traffic.txt),
    or None when there is none or the kernel sources have changed since the counters were taken."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    sha, val, most = None, None, -1
    for line in open(path):
        if line.startswith("source_sha1"):
            sha = line.split()[1]
        elif not line.startswith("#") and "|" in line:
            w, k, f, wr, disp = [x.strip() for x in line.split("|")]
            # several instantiations may match: the one with the most dispatches is the one that carries the time
            if w == workload and k.startswith(kernel_prefix) and int(disp.split()[1]) > most:
                most = int(disp.split()[1])
                val = (float(f.split()[1]) + float(wr.split()[1])) * 1024.0
    return val if sha == source_sha1() else None


def time_steps(ex, torch, d, out, tol, steps, warmup, norm=0):
    for _ in range(warmup):
        ex.expm(d, tol, out=out, norm=norm)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        ex.expm(d, tol, out=out, norm=norm)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms / steps, e0.elapsed_time(e1) / steps


def time_steps_graph(ex, torch, d, out, tol, steps, norm=0):
    """The same `steps` calls replayed from HIP graphs of up to 20 calls each (single-launch path only): what a
    caller with a launch-bound loop does; takes the host's per-call cost out of the measurement.  None if the
    capture fails."""
    calls = max(c for c in range(1, 21) if steps % c == 0)
    try:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for _ in range(calls):
                ex.expm(d, tol, out=out, norm=norm)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps // calls):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / steps
        del graph
        return ms, calls
    except Exception as e:  # noqa: BLE001 - any failure of the capture leaves the eager figure standing
        print("bench.py: graph capture failed (%s); eager launches only" % e, file=sys.stderr)
        return None


def kernel_profile(ex, torch, d, out, tol, steps, norm=0):
    """Per-kernel-class time from HIP events recorded around every launch on the launch stream."""
    ex.expm_profile_reset()
    ex.expm_profile_enable(True)
    for _ in range(steps):
        ex.expm(d, tol, out=out, norm=norm)
    torch.cuda.synchronize()
    prof = ex.expm_profile_read()
    ex.expm_profile_enable(False)
    ex.expm_profile_reset()
    return prof


def time_select(ex, torch, d, tol, steps):
    ex.expm_select(d, tol)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ex.expm_select(d, tol)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def small_matrix_context(ex, torch, workloads, name, d, out, norm):
    """Figures that put the HBM fraction of a 4096-matrix batch in context: what a plain device copy of the same
    bytes takes (launch and latency floor of any kernel on so little data), and the same kernel on a batch 64
    times larger (same recipe and seed), where it runs at its own instruction rate."""
    w = workloads.WORKLOADS[name]
    reps = 200
    for _ in range(10):
        out.copy_(d)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        out.copy_(d)
    e1.record()
    torch.cuda.synchronize()
    copy_ms = e0.elapsed_time(e1) / reps
    big = 64 * w.batch
    ab = torch.from_numpy(workloads.make_workload(name, batch=big)).cuda()
    ob = torch.empty_like(ab)
    for _ in range(3):
        ex.expm(ab, w.tol, out=ob, norm=norm)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(20):
        ex.expm(ab, w.tol, out=ob, norm=norm)
    e1.record()
    torch.cuda.synchronize()
    big_ms = e0.elapsed_time(e1) / 20
    nbytes = 2.0 * ab.numel() * ab.element_size()
    del ab, ob
    ex.expm(d, w.tol, out=out, norm=norm)  # leave the workload itself as the last call
    torch.cuda.synchronize()
    return {"device_copy_same_bytes_ms": copy_ms,
            "batch_x64": {"batch": big, "ms_per_step": big_ms, "matrices_per_s": big / (big_ms * 1e-3),
                          "hbm_gbs": nbytes / (big_ms * 1e-3) / 1e9, "hbm_frac": nbytes / (big_ms * 1e-3) / 1e9 / PEAK["hbm"]}}


def run_lowrank_workload(name, steps, warmup, with_cpu):
    """Low-rank variant (Sec. 2.2): e^(A1 A2) = I + A1 phi(A2 A1) A2."""
    import numpy as np
    import torch
    import paper_2512_20777_amd as ex
    from paper_2512_20777_amd import workloads
    w = workloads.LOWRANK_WORKLOADS[name]
    a1, a2 = workloads.make_lowrank_workload(name)
    d1, d2 = torch.from_numpy(a1).cuda(), torch.from_numpy(a2).cuda()
    n, t, batch = w["n"], w["t"], w["batch"]
    out = torch.empty((batch, n, n), dtype=d1.dtype, device="cuda")
    tol = 2.0 ** -24 if w["dtype"] == "f32" else 2.0 ** -53
    for _ in range(warmup):
        ex.expm_lowrank(d1, d2, tol, out=out)
    torch.cuda.synchronize()
    stats = ex.expm_get_stats()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        ex.expm_lowrank(d1, d2, tol, out=out)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    psteps = max(2, min(steps, 20))
    ex.expm_profile_reset()
    ex.expm_profile_enable(True)
    for _ in range(psteps):
        ex.expm_lowrank(d1, d2, tol, out=out)
    torch.cuda.synchronize()
    prof = ex.expm_profile_read()
    ex.expm_profile_enable(False)
    ex.expm_profile_reset()
    wb = 4 if w["dtype"] == "f32" else 8
    algo_bytes = batch * (n * n + 2.0 * n * t) * wb                 # read A1, A2, write e^W
    flops = batch * (2.0 * t * t * n * 2 + 2.0 * n * n * t) + 2.0 * t ** 3 * stats["products"]
    # The three rectangular products (V = A2 A1, U = A1 phi, U A2 + I) carry the time; the last one does 2t flops per
    # output element, which at t = 64 in fp32 is above the ridge of the two roofs (19.7 flop/byte): matrix-core bound.
    k = prof["gemm"]
    peak = PEAK["mfma_f64" if w["dtype"] == "f64" else "mfma_f32"]
    ach = k["flops"] / (k["ms"] * 1e-3) / 1e12
    res = {"workload": name, "n": n, "t": t, "batch": batch, "dtype": w["dtype"], "tol": tol, "norm": "one",
           "steps": steps, "warmup": warmup, "ms_per_step": wall_ms, "ms_per_step_events": e0.elapsed_time(e1) / steps,
           "matrices_per_s": batch / (wall_ms * 1e-3), "tflops": flops / (wall_ms * 1e-3) / 1e12,
           "products": stats["products"], "rounds": 0,
           "hist_m": {str(kk): v for kk, v in stats["hist_m"].items() if v}, "hist_s": {"0": batch},
           "select_ms": None,
           "kernel_ms_per_step": {kk: v["ms"] / psteps for kk, v in prof.items() if v["launches"]},
           "roofline": {"bound": "mfma", "kernel": "rect_gemm_kernel", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                        "frac": ach / peak, "traffic": None, "avg_launch_ms": k["ms"] / k["launches"],
                        "launches_per_step": k["launches"] / psteps, "whole_call_frac": flops / (wall_ms * 1e-3) / 1e12 / peak,
                        "hbm_gbs_whole_call": algo_bytes / (wall_ms * 1e-3) / 1e9}}
    # HBM bytes of the last product (the 128x128-tile instantiation), which carries most of the time
    res["roofline"]["traffic"] = recorded_traffic(name, "rect_gemm_kernel<%s, 4" % ("float" if w["dtype"] == "f32" else "double"))
    if with_cpu:
        from oracle import oracle_lowrank_batch
        sub = min(batch, 8)
        oracle_lowrank_batch(a1[:1], a2[:1], tol)
        t0 = time.perf_counter()
        _, info = oracle_lowrank_batch(a1[:sub], a2[:sub], tol)
        sec = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": sub / sec, "unit": "matrices/s", "cores": int(info["threads"]), "kind": "oracle",
                               "sample": "first %d pairs of the batch, one run, %.2f s" % (sub, sec)}
    return res


def cpu_baseline(name, a, tol, workloads, ms=None):
    """The oracle, as it stands, on the host cores, timed in this run: the whole batch when that takes seconds; for the
    4096 x 4096 workloads (whose whole run takes minutes) the first matrix of the batch, scaled by the number of
    products the oracle spends on the whole batch.  `ms` = (m, s) per matrix as the device selected them."""
    import numpy as np
    from oracle import oracle_expm_batch
    w = workloads.WORKLOADS[name]
    if name.startswith("C5"):
        # The oracle forms W^2 for the selection, then sums the series term by term from A (m - 1 products, one more
        # for the b16 A^16 term of 15+) and squares s times: per matrix 1 + (m - 1) + [m = 15] + s products of
        # 2 n^3 flops, everything else is O(n^2).
        m, sc = ms
        counts = [1 + max(int(mm) - 1, 0) + (1 if mm == 15 else 0) + int(ss) for mm, ss in zip(m, sc)]
        # sample: the whole oracle on the first matrix of the batch (the one with the smallest norm, no squarings)
        t0 = time.perf_counter()
        _, info = oracle_expm_batch(a[:1], tol)
        sec = time.perf_counter() - t0
        used = int(info["threads"])
        own = 1 + max(int(info["m"][0]) - 1, 0) + (1 if info["m"][0] == 15 else 0) + int(info["s"][0])
        total = sec * sum(counts) / own
        res = {"value": w.batch / total, "unit": "matrices/s", "cores": used, "kind": "oracle",
               "sample": "the oracle on the first matrix of the batch, timed in this run: %.1f s for its %d products of "
                         "4096^3 on %d threads; the batch costs the oracle %d products (1 + (m-1) + [m=15] + s per "
                         "matrix), i.e. %.0f s, extrapolated by product count" % (sec, own, used, sum(counts), total)}
        path = os.path.join(ROOT, "tests", "golden", "c5_samples_%s.npz" % w.dtype)
        if os.path.exists(path):
            g = np.load(path)
            res["whole_batch_recorded"] = {"seconds": float(g["oracle_seconds"][0]), "cores": int(g["oracle_threads"][0]),
                                           "note": "the oracle's full run when tests/golden/make_c5_samples.py wrote the "
                                                   "stored samples, on another machine"}
        return res
    reps = {"F1": 50, "C1": 200, "C2": 50, "C3": 5, "C4": 3}[name]
    if w.norm == "inf":  # infinity-norm selection of W = 1-norm selection of its transpose (same work for the oracle)
        a = np.ascontiguousarray(np.swapaxes(a, -1, -2))
    oracle_expm_batch(a[: max(1, min(4, a.shape[0]))], tol)  # load the library, warm caches
    t0 = time.perf_counter()
    used = 0
    for _ in range(reps):
        _, info = oracle_expm_batch(a, tol)
        used = info["threads"]
    sec = (time.perf_counter() - t0) / reps
    res = {"value": a.shape[0] / sec, "unit": "matrices/s", "cores": int(used), "kind": "oracle",
           "sample": "whole batch of %d, mean of %d runs in this run, %.4f s per batch" % (a.shape[0], reps, sec)}
    if name in ("C1", "C2", "F1"):
        # the small workloads also on one core (a threaded run of so little work mostly measures the thread team)
        r1 = max(1, reps // 5)
        t0 = time.perf_counter()
        for _ in range(r1):
            oracle_expm_batch(a, tol, threads=1)
        res["one_core_value"] = a.shape[0] / ((time.perf_counter() - t0) / r1)
    return res


def run_workload(name, steps, warmup, with_cpu, extras=False, compare_ps=False):
    import numpy as np
    import torch
    import paper_2512_20777_amd as ex
    from paper_2512_20777_amd import workloads

    w = workloads.WORKLOADS[name]
    a = workloads.make_workload(name)
    d = torch.from_numpy(a).cuda()
    out = torch.empty_like(d)
    ex.expm_reserve(w.n, w.batch, ex.DTYPE_F64 if w.dtype == "f64" else ex.DTYPE_F32)
    norm = ex.NORM_INF if w.norm == "inf" else ex.NORM_ONE
    ex.expm(d, w.tol, out=out, norm=norm)
    torch.cuda.synchronize()
    stats = ex.expm_get_stats()
    wall_ms, ev_ms = time_steps(ex, torch, d, out, w.tol, steps, warmup, norm)
    launch, eager_ms = "eager", wall_ms
    if stats["fused_path"] and ev_ms < 0.05:
        # a step of a few microseconds is bounded by the host's launch rate: time the same steps from HIP graphs
        # too and take the faster of the two ways of launching them
        g = time_steps_graph(ex, torch, d, out, w.tol, steps, norm)
        if g is not None and g[0] < wall_ms:
            wall_ms, launch = g[0], "hip graph, %d steps per graph" % g[1]
    prof = kernel_profile(ex, torch, d, out, w.tol, max(2, min(steps, 20)), norm)
    sel_ms = time_select(ex, torch, d, w.tol, max(2, min(steps, 20))) if extras else None

    wbytes = 8 if w.dtype == "f64" else 4
    flops = 2.0 * w.n ** 3 * stats["products"]          # products the selection asked for, W^2 counted once
    algo_bytes = 2.0 * w.batch * w.n * w.n * wbytes      # read W, write e^W
    res = {
        "workload": name, "n": w.n, "batch": w.batch, "dtype": w.dtype, "tol": w.tol, "norm": w.norm,
        "steps": steps, "warmup": warmup,
        "ms_per_step": wall_ms, "ms_per_step_events": ev_ms, "launch": launch, "ms_per_step_eager": eager_ms,
        "matrices_per_s": w.batch / (wall_ms * 1e-3),
        "tflops": flops / (wall_ms * 1e-3) / 1e12,
        "products": stats["products"], "rounds": stats["rounds"],
        "hist_m": {str(k): v for k, v in stats["hist_m"].items() if v},
        "hist_s": {str(i): v for i, v in enumerate(stats["hist_s"]) if v},
        "select_ms": sel_ms,
        "kernel_ms_per_step": {k: v["ms"] / max(2, min(steps, 20)) for k, v in prof.items() if v["launches"]},
    }
    if stats["fused_path"]:
        # a step is exactly one launch of this kernel: its average duration is the timed region over the steps
        # (events on the launch stream around the eager steps, or the graph-launched steps when those were faster;
        # a pair of events around every single launch, as the per-class timers record, would add the launch gap
        # to a kernel of a few microseconds)
        avg_ms = min(ev_ms, wall_ms)
        # one-tile fp64 matrices run in the register-resident kernel, everything else fused in the LDS kernel
        fused_name = "fused_tile_kernel" if (w.n <= 16 and w.dtype == "f64") else "fused_expm_kernel"
        peak = PEAK["mfma_f64" if w.dtype == "f64" else "mfma_f32"]
        ridge = peak * 1e12 / (PEAK["hbm"] * 1e9)          # flop per byte where the two roofs meet
        if flops / algo_bytes >= ridge:                     # dense contraction dominates (n of order 100)
            ach = flops / (avg_ms * 1e-3) / 1e12
            res["roofline"] = {"bound": "mfma", "kernel": fused_name, "achieved": ach, "peak": peak,
                               "unit": "TFLOP/s", "frac": ach / peak, "traffic": None, "avg_launch_ms": avg_ms,
                               "hbm_gbs_in_kernel": algo_bytes / (avg_ms * 1e-3) / 1e9,
                               "whole_call_frac": res["tflops"] / peak}
        else:
            ach = algo_bytes / (avg_ms * 1e-3) / 1e9
            res["roofline"] = {"bound": "hbm", "kernel": fused_name, "achieved": ach, "peak": PEAK["hbm"],
                               "unit": "GB/s", "frac": ach / PEAK["hbm"], "traffic": None, "avg_launch_ms": avg_ms,
                               "mfma_tflops_in_kernel": flops / (avg_ms * 1e-3) / 1e12}
    else:
        k = prof["gemm"]
        peak = PEAK["mfma_f64" if w.dtype == "f64" else "mfma_f32"]
        ach = k["flops"] / (k["ms"] * 1e-3) / 1e12       # 2 n^3 per launched product / summed launch time
        res["roofline"] = {"bound": "mfma", "kernel": "gemm_round_kernel", "achieved": ach, "peak": peak,
                           "unit": "TFLOP/s", "frac": ach / peak, "traffic": None,
                           "avg_launch_ms": k["ms"] / k["launches"], "launches_per_step": k["launches"] / max(2, min(steps, 20)),
                           "whole_call_frac": res["tflops"] / peak}
    res["roofline"]["traffic"] = recorded_traffic(name, res["roofline"]["kernel"])
    if compare_ps:
        # the paper's own comparison (Sec. 4): same tolerance, Paterson-Stockmeyer evaluation + Algorithm 3
        ps_steps = max(2, steps // 4)
        for _ in range(2):
            ex.expm(d, w.tol, out=out, scheme=ex.SCHEME_PS, norm=norm)
        torch.cuda.synchronize()
        ps_stats = ex.expm_get_stats()
        t0 = time.perf_counter()
        for _ in range(ps_steps):
            ex.expm(d, w.tol, out=out, scheme=ex.SCHEME_PS, norm=norm)
        torch.cuda.synchronize()
        ps_ms = (time.perf_counter() - t0) * 1e3 / ps_steps
        res["paterson_stockmeyer_variant"] = {
            "ms_per_step": ps_ms, "products": ps_stats["products"],
            "product_ratio_vs_main": ps_stats["products"] / max(1, stats["products"]),
            "time_ratio_vs_main": ps_ms / wall_ms,
            "hist_m": {str(k): v for k, v in ps_stats["hist_m"].items() if v}}
        if True:
            # the paper's baseline (its Algorithm 1): on chip for the small sizes, term rounds above
            for _ in range(2):
                ex.expm(d, w.tol, out=out, scheme=ex.SCHEME_BASELINE, norm=norm)
            torch.cuda.synchronize()
            b_stats = ex.expm_get_stats()
            t0 = time.perf_counter()
            for _ in range(ps_steps):
                ex.expm(d, w.tol, out=out, scheme=ex.SCHEME_BASELINE, norm=norm)
            torch.cuda.synchronize()
            b_ms = (time.perf_counter() - t0) * 1e3 / ps_steps
            res["baseline_algorithm1"] = {
                "ms_per_step": b_ms, "products_as_priced_by_the_paper": b_stats["products"],
                "product_ratio_vs_main": b_stats["products"] / max(1, stats["products"]),
                "time_ratio_vs_main": b_ms / wall_ms}
        ex.expm(d, w.tol, out=out, norm=norm)  # leave the main scheme as the last call
        torch.cuda.synchronize()
    if extras and stats["fused_path"] and res["roofline"]["bound"] == "hbm":
        res["context"] = small_matrix_context(ex, torch, workloads, name, d, out, norm)
    if with_cpu:
        ms = None
        if name.startswith("C5"):
            m_sel, s_sel, _ = ex.expm_select(d, w.tol, norm=norm)
            ms = (m_sel, s_sel)
        res["cpu_baseline"] = cpu_baseline(name, a, w.tol, workloads, ms)
    del d, out
    torch.cuda.empty_cache()
    return res


def pmc_pass(name, steps):
    """A few steps of one workload and a 256 MiB device-to-device copy (the counter calibration)."""
    import torch
    import paper_2512_20777_amd as ex
    from paper_2512_20777_amd import workloads
    if name in workloads.LOWRANK_WORKLOADS:
        a1, a2 = workloads.make_lowrank_workload(name)
        d1, d2 = torch.from_numpy(a1).cuda(), torch.from_numpy(a2).cuda()
        for _ in range(steps):
            ex.expm_lowrank(d1, d2)
    else:
        w = workloads.WORKLOADS[name]
        d = torch.from_numpy(workloads.make_workload(name)).cuda()
        out = torch.empty_like(d)
        norm = ex.NORM_INF if w.norm == "inf" else ex.NORM_ONE
        for _ in range(steps):
            ex.expm(d, w.tol, out=out, norm=norm)
    torch.cuda.synchronize()
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")   # 256 MiB
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"pmc_pass": name, "steps": steps, "copy_bytes_each_way": src.numel() * 4}))
    ex.expm_shutdown()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0)
    ap.add_argument("--warmup", type=int, default=-1)
    ap.add_argument("--workload", default="C5f64")
    ap.add_argument("--no-others", action="store_true", help="only the headline workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--pmc-pass", action="store_true", help="short run for hardware-counter collection: a few "
                    "steps of the workload plus a plain device copy of 256 MiB as the calibration kernel")
    ap.add_argument("--compare-ps", "--compare", dest="compare_ps", action="store_true",
                    help="also run the paper's two comparison schemes (Paterson-Stockmeyer; its Algorithm 1 baseline "
                    "where available) and report their products and time relative to the main scheme")
    ap.add_argument("--no-extras", dest="extras", action="store_false",
                    help="only the timed steps and the per-class timers: no timing of expm_select() alone, no "
                    "context figures (device copy, graph replay, larger batch).  Those add launches of the same "
                    "kernels that are not expm() steps of the workload, so kernel traces taken for per-kernel "
                    "averages leave them out")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library runs on one GPU; --gpus %d is not supported (batches shard across GPUs "
              "with no communication, one process per GPU, each running this same benchmark)" % args.gpus,
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    import paper_2512_20777_amd as ex
    ex.load_library()

    head = args.workload
    if args.pmc_pass:
        pmc_pass(head, args.steps if args.steps > 0 else 3)
        return
    from paper_2512_20777_amd import workloads
    lowrank_head = head in workloads.LOWRANK_WORKLOADS
    steps = args.steps if args.steps > 0 else DEFAULT_STEPS.get(head, 20)
    warmup = args.warmup if args.warmup >= 0 else DEFAULT_WARMUP.get(head, 5)
    if lowrank_head:
        main_res = run_lowrank_workload(head, steps, warmup, not args.no_cpu)
    else:
        main_res = run_workload(head, steps, warmup, not args.no_cpu, args.extras, args.compare_ps)
    per = [main_res]
    if not args.no_others:
        for name in ("C1", "C2", "C3", "C4", "C5f64", "C5f32", "F1"):
            if name == head:
                continue
            per.append(run_workload(name, DEFAULT_STEPS[name], DEFAULT_WARMUP[name], not args.no_cpu, args.extras,
                                    args.compare_ps))
        if not lowrank_head:
            per.append(run_lowrank_workload("L1", DEFAULT_STEPS["L1"], DEFAULT_WARMUP["L1"], not args.no_cpu))
        per.sort(key=lambda r: r["workload"])
    note = workloads.LOWRANK_WORKLOADS[head]["note"] if lowrank_head else workloads.WORKLOADS[head].note
    line = {
        "metric": "matrix exponentials/sec + achieved TFLOP/s (% of MFMA peak) per (n,batch,dtype)",
        "value": main_res["matrices_per_s"], "unit": "matrices/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res["dtype"], "data": "synthetic",
        "config": {"workload": "%s: %s" % (head, note), "launch": main_res.get("launch", "eager"), "n": main_res["n"],
                   "batch": main_res["batch"], "tol": main_res["tol"], "norm": main_res["norm"]},
        "tflops": main_res["tflops"],
        "roofline": {k: main_res["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "traffic")},
        "cpu_baseline": main_res.get("cpu_baseline"),
        "per_config": per,
    }
    print(json.dumps(line))
    ex.expm_shutdown()


if __name__ == "__main__":
    main()
