#!/usr/bin/env python3
"""Benchmark of the fused SDDMM-SpMM kernel on one MI355X.

A step is one fusedmm_execute call (the whole hot path: schedule lookup, gather,
VOP/ROP/SOP/MOP/AOP, store, split-row merge) over one synthetic workload whose
inputs already sit in HBM.  Prints ONE JSON line.

    python bench.py [--workload c5] [--steps K] [--warmup W] [--gpus 1]

The default workload is c5, the largest configuration that fits one GPU (Y = 4 GiB, far
beyond the caches).  Without --workload the same line also carries, under
config.all_workloads, value / ms_per_step / kernel_ms / parity for c2, c3 and c4.

Metric: G(edge*dim)/s = nnz * d / seconds per step.  The roofline object prices the bytes
the main kernel really moved between the L2s and the memory fabric (rocprofv3 FETCH_SIZE +
WRITE_SIZE per launch, taken from profiles/hbm_traffic_per_launch.txt when that table was
measured on this very build and plan) against the 8 TB/s HBM peak: a fraction that cannot
exceed 1.  The algorithmic rate (the paper's "no reuse of Y rows" byte model, Section IV-C)
is reported beside it as algorithmic_GBs / algorithmic_over_peak; it exceeds the peak when
the caches serve repeated rows.  cpu_baseline times the unfused CPU oracle (fp32 build).
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")


def kernel_sources_sha16() -> str:
    """Identifies the build the traffic table belongs to: a hash of the library's sources."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2011_06391_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.startswith("fusedmm_") and name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, plan_stats: dict):
    """L2 <-> fabric bytes per launch of the main kernel from the tracked table, if the table's row was
    measured with these kernel sources and this plan; else (None, None, why).  Rows: workload, sources
    hash, partial rows, tile segments, column classes, fetch bytes, write bytes, L2 hit rate, commit."""
    if not os.path.exists(TRAFFIC_TABLE):
        return None, None, "no traffic table (profiles/hbm_traffic_per_launch.txt)"
    sha = kernel_sources_sha16()
    why = f"no row for workload {workload}"
    for line in open(TRAFFIC_TABLE):
        f = line.split("#")[0].split()
        if len(f) < 9 or f[0] != workload:
            continue
        if f[1] != sha:
            why = f"stale: the table's {workload} row was measured on kernel sources {f[1]}, this build is {sha}"
            continue
        if (int(f[2]), int(f[3]), int(f[4])) != (plan_stats["partials"], plan_stats["tile_segments"],
                                                 plan_stats["column_classes"]):
            why = f"stale: the table's {workload} row was measured with another plan"
            continue
        src = (f"profiles/hbm_traffic_per_launch.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per launch, calibrated "
               f"with the copy kernel; measured at commit {f[8]}, kernel sources {sha}")
        return int(f[5]) + int(f[6]), float(f[7]), src
    return None, None, why


def parity_sample(w, rows, Z_rows, aop="SUM"):
    """Part of the CPU leg: the fp64 oracle recomputes a sample of rows of the timed result."""
    import numpy as np
    import oracle

    sub = w.csr.take_rows(rows)
    if aop == "SUM":
        Zr, S, _ = oracle.unfused(sub.rowptr, sub.colidx, sub.values, w.X[rows], w.Y, w.pattern)
    else:
        Zr, S, _ = oracle.unfused_general(sub.rowptr, sub.colidx, sub.values, w.X[rows], w.Y, oracle.PATTERNS[w.pattern],
                                          {"MAX": "AMAX", "MIN": "AMIN", "MEAN": "AMEAN"}[aop])
    err, _, viol = oracle.compare(Z_rows, Zr, S)
    return {"rows_checked": int(len(rows)), "stored_entries_checked": int(sub.nnz), "max_rel_err": err,
            "tolerance": 1e-4, "nonzero_where_all_terms_zero": viol,
            "rule": "max |Z_gpu - Z_oracle| / sum|terms| over the sampled rows (longest rows + random rows)"}


def cpu_baseline(w, budget_edges_dim: float = 6.0e10):
    """Time the oracle's fp32 two-phase (unfused) build on a bounded sample of the rows."""
    import numpy as np
    import oracle
    from paper_2011_06391_amd import synth

    g = w.csr
    work = g.nnz * w.d
    if work <= budget_edges_dim:
        sub, rows, sample = g, None, "whole workload"
    else:
        frac = budget_edges_dim / work
        rng = np.random.default_rng(2024)
        rows = np.sort(rng.choice(g.m, max(1, int(g.m * frac)), replace=False)).astype(np.int64)
        sub = g.take_rows(rows)
        sample = f"{len(rows)} random rows of {g.m} ({sub.nnz} of {g.nnz} stored entries), all of Y"
    X = w.X if rows is None else w.X[rows]
    # about 10 s of CPU work: the sample is run once, then repeated until ~10 s have been spent
    # (at most 400 runs); the median run is reported
    times = []
    spent, reps = 0.0, 0
    while reps < 400 and (reps == 0 or spent + times[0] <= 10.0):
        t0 = time.perf_counter()
        oracle.unfused(sub.rowptr, sub.colidx, sub.values, X, w.Y, w.pattern, precision="f32", want_abs=False)
        times.append(time.perf_counter() - t0)
        spent += times[-1]
        reps += 1
    t = sorted(times)[len(times) // 2]
    return {"value": sub.nnz * w.d / t / 1e9, "unit": "G(edge*dim)/s", "cores": synth.num_threads(),
            "kind": "oracle", "sample": sample, "seconds": t, "repetitions": reps, "cpu_seconds_spent": spent, "precision": "fp32 unfused two-phase"}


def run(workload: str, steps: int, warmup: int, with_cpu: bool, options=None, d=None, copy_mib: int = 0,
        autotune: bool = False, y_storage: str = "f32", with_context: bool = True, relabel: bool = True,
        time_cpu: bool = True, aop: str = "SUM"):
    import torch
    from paper_2011_06391_amd import binding, model, synth

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (torch.cuda.is_available() is False)")
    binding.load()
    torch.cuda.set_device(0)
    t0 = time.perf_counter()
    w = synth.make_workload(workload, d=d, relabel=relabel)
    g = w.csr
    gen_s = time.perf_counter() - t0

    rp = torch.from_numpy(g.rowptr).cuda()
    ci = torch.from_numpy(g.colidx).cuda()
    Xd = torch.from_numpy(w.X).cuda()
    Yd = Xd if w.Y is w.X else torch.from_numpy(w.Y).cuda()
    vd = None if g.values is None else torch.from_numpy(g.values).cuda()
    f64 = y_storage == "f64"   # everything in double precision (secondary measurement)
    if f64:
        Xd = Xd.double()
        Yd = Xd if w.Y is w.X else Yd.double()
        vd = None if vd is None else vd.double()
        with_context = False
    Z = torch.empty((g.m, w.d), dtype=torch.float64 if f64 else torch.float32, device="cuda")
    uses_x = w.pattern != "gcn"
    ops = binding.fusedmm_ops_preset(w.pattern)
    ops.aop = binding.AOP[aop]   # the pattern's messages pooled another way (secondary measurements)

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    custom_plan = bool(options)
    options = dict(options or {})
    options.setdefault("feature_dim_hint", 2 * w.d if f64 else w.d)   # the hint counts 4-byte elements
    if autotune and not f64:
        plan = binding.Plan.tuned(g.m, g.n, rp, ci, ops, Xd if uses_x else None, Yd, Z, vd)
        options = plan.tuned_options
    else:
        plan = binding.Plan(g.m, g.n, rp, ci, options)
    if f64:
        plan.reserve_f64(w.d)
    else:
        plan.reserve(w.d)
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t0) * 1e3
    if y_storage == "f32":   # inspection + the very first execute, as one figure (context, never part of `value`)
        plan.execute(ops, Xd if uses_x else None, Yd, Z, vd)
        torch.cuda.synchronize()
    plan_plus_first_execute_ms = (time.perf_counter() - t0) * 1e3

    Yb = None
    y_bf16 = y_storage in ("bf16", "f16")  # any 2-byte storage of Y
    if y_bf16:  # optional storage mode, never the default: Y rounded once to bfloat16 / half, arithmetic stays fp32
        Yb = torch.empty((g.n, w.d), dtype=torch.int16, device="cuda")
        (binding.fusedmm_to_bf16 if y_storage == "bf16" else binding.fusedmm_to_f16)(Yb, Yd, g.n * w.d)
        torch.cuda.synchronize()

    # one step = one fusedmm_execute[_bf16y|_f16y] call; the arguments are marshalled once, outside the loop
    step = plan.bind(ops, Xd if uses_x else None, Yb if Yb is not None else Yd, Z, vd, y_format=y_storage)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: exactly `steps` executes, nothing else on the stream
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    # the same `steps` executes again, now with HIP events recorded around the main kernel on
    # the launch stream (the two event records per step cost ~4 us of stream time, which is why
    # they are kept out of the region that defines `value`; the kernel's own duration is the same)
    plan.set_profiling(True)
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    samples, empties = plan.read_profile_samples()
    kernel_ms_sum, empty_ms_sum, calls = sum(samples), sum(empties), len(samples)
    plan.set_profiling(False)
    assert torch.isfinite(Z[: min(g.m, 4096)]).all().item()
    deg = g.degrees()
    import numpy as np
    sample_rows = np.unique(np.concatenate([np.argsort(-deg)[:4], np.random.default_rng(7).choice(g.m, min(g.m, 512),
                                                                                                 replace=False)]))
    Z_sample = Z[torch.from_numpy(sample_rows).cuda()].cpu().numpy()  # rows of the timed result, checked on the CPU leg

    ms_per_step = elapsed * 1e3 / steps
    tr = model.traffic(g.m, g.n, g.nnz, w.d, uses_x, vd is not None, w.Y is w.X, y_bytes=2 if y_bf16 else 0,
                       elem_bytes=8 if f64 else 4)
    kernel_ms = (kernel_ms_sum - empty_ms_sum) / max(1, calls)  # bracket cost measured by an empty bracket per call
    if kernel_ms <= 0.0:  # a kernel of a few microseconds can vanish in the bracket's own jitter
        kernel_ms = kernel_ms_sum / max(1, calls)
    kernel_s = kernel_ms * 1e-3
    stats = plan.stats()
    if y_bf16 or f64 or not relabel:
        traffic_bytes, l2_hit, traffic_source = None, None, "not measured for this storage mode / vertex order"
    else:
        traffic_bytes, l2_hit, traffic_source = measured_traffic(workload if not d else f"{workload}:d{w.d}", stats)
    # the priced bytes: what the kernel moved beyond the L2s when that was measured on this build and plan,
    # else the compulsory bytes (every array once), a lower bound of it; both keep the fraction below 1
    priced = traffic_bytes if traffic_bytes is not None else tr.min_bytes
    basis = ("measured L2<->fabric bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated)"
             if traffic_bytes is not None else "compulsory bytes (every array moved once): a lower bound of the traffic")
    achieved = priced / kernel_s / 1e9
    out = {
        "metric": "fused SDDMM-SpMM throughput: G(edge*dim)/s + achieved HBM GB/s vs peak, 1 GPU",
        "value": g.nnz * w.d / (ms_per_step * 1e-3) / 1e9,
        "unit": "G(edge*dim)/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": f"f32 (Y stored as {y_storage})" if y_bf16 else y_storage, "data": "synthetic",
        "config": {"workload": workload, "description": w.description, "pattern": w.pattern, "aop": aop,
                   "vertex_order": "seeded random permutation" if relabel else "as generated (natural order)",
                   "n": g.m, "nnz": g.nnz, "d": w.d, "max_degree": int(deg.max()),
                   "empty_rows": int((deg == 0).sum()), "plan": stats, "plan_ms": plan_ms,
                   "plan_plus_first_execute_ms": plan_plus_first_execute_ms, "plan_options": options, "autotuned": autotune,
                   "workspace_bytes": plan.workspace_bytes(w.d), "generate_s": gen_s,
                   "kernel_sources_sha16": kernel_sources_sha16()},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": model.MI355X_HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / model.MI355X_HBM_PEAK_GBS, "achieved_basis": basis,
                     "traffic": traffic_bytes, "traffic_source": traffic_source, "l2_hit_rate": l2_hit,
                     "algorithmic_bytes": tr.model_bytes, "algorithmic_GBs": tr.model_bytes / kernel_s / 1e9,
                     "algorithmic_over_peak": tr.model_bytes / kernel_s / 1e9 / model.MI355X_HBM_PEAK_GBS,
                     "compulsory_bytes": tr.min_bytes, "compulsory_GBs": tr.min_bytes / kernel_s / 1e9,
                     "kernel": "fusedmm_fast_kernel", "kernel_ms": kernel_ms,
                     "kernel_timing": "HIP events around the main kernel on the launch stream, same K executes repeated "
                                      "right after the timed region; an empty event bracket per call is subtracted",
                     "kernel_ms_with_bracket": kernel_ms_sum / max(1, calls),
                     "kernel_ms_median": (sorted(samples)[len(samples) // 2] - sorted(empties)[len(empties) // 2])
                     if samples else None,
                     "kernel_ms_min": (min(samples) - sorted(empties)[len(empties) // 2]) if samples else None,
                     "bytes_per_edge": tr.per_edge_bytes, "bytes_per_row": tr.per_row_bytes},
    }
    # Context figures, measured after and outside the timed region (never part of `value`):
    # the same step replayed from a HIP graph (launch overhead removed), and the streaming
    # bandwidth of a plain copy kernel on this machine (read + write bytes per second).
    context = {}
    try:
        if not with_context:
            raise RuntimeError("skipped (--no-context)")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):  # bound inside the capture: the current stream is the capturing one here
            plan.bind(ops, Xd if uses_x else None, Yb if Yb is not None else Yd, Z, vd, y_format=y_storage)()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        context["ms_per_step_hip_graph"] = (time.perf_counter() - t0) * 1e3 / steps
        del graph
    except Exception as exc:  # context only: never let it break the benchmark line
        context["hip_graph_error"] = repr(exc)[:200]
    try:
        if not with_context:
            raise RuntimeError("skipped (--no-context)")
        nbytes = 1 << 30
        src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        binding.fusedmm_debug_copy(dst, src, nbytes)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            binding.fusedmm_debug_copy(dst, src, nbytes)
        e1.record()
        torch.cuda.synchronize()
        context["copy_kernel_GBs_read_plus_write"] = 5 * 2 * nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del src, dst
    except Exception as exc:
        context["copy_error"] = repr(exc)[:200]
    try:
        if not with_context:
            raise RuntimeError("skipped (--no-context)")
        # the gather ceiling of this graph and schedule: the GCN pattern with unit edge values is the
        # same stream of row gathers with one FMA per element and no ROP / SOP
        ones = torch.ones(max(1, g.nnz), dtype=torch.float32, device="cuda")
        gcn = binding.fusedmm_ops_preset("gcn")
        for _ in range(3):
            plan.execute(gcn, None, Yd, Z, ones)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            plan.execute(gcn, None, Yd, Z, ones)
        torch.cuda.synchronize()
        context["ms_per_step_pure_gather_same_schedule"] = (time.perf_counter() - t0) * 1e3 / steps
        del ones
    except Exception as exc:
        context["gather_error"] = repr(exc)[:200]
    try:
        if not with_context:
            raise RuntimeError("skipped (--no-context)")
        # cold caches: 512 MiB are streamed through L2 and Infinity Cache before every execute;
        # only the main kernel is timed (events), 20 times
        fl_src = torch.ones(128 << 20, dtype=torch.float32, device="cuda")
        fl_dst = torch.empty_like(fl_src)
        plan.set_profiling(True)
        for _ in range(20):
            binding.fusedmm_debug_copy(fl_dst, fl_src, 512 << 20)
            step()
        torch.cuda.synchronize()
        ms_sum, empty_sum, n_calls = plan.read_profile()
        plan.set_profiling(False)
        context["main_kernel_ms_cold_caches"] = (ms_sum - empty_sum) / max(1, n_calls)
        del fl_src, fl_dst
    except Exception as exc:
        context["cold_error"] = repr(exc)[:200]
    out["config"]["context"] = context
    if copy_mib > 0:
        # one launch of the plain copy kernel with known traffic, for calibrating profiler counters
        src = torch.ones(copy_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        binding.fusedmm_debug_copy(dst, src, copy_mib << 20)
        torch.cuda.synchronize()
        assert (dst[-4:] == 1).all().item()
        out["config"]["copy_calibration_bytes_each_way"] = copy_mib << 20
        del src, dst
    plan.close()
    del Z, Xd, Yd, rp, ci
    torch.cuda.empty_cache()
    if with_cpu:
        out["cpu_baseline"] = cpu_baseline(w) if time_cpu else {}
        if not y_bf16:  # the oracle would have to be fed the rounded Y; tests/test_reduced_storage_gpu.py does that
            out["cpu_baseline"]["parity_of_timed_result"] = parity_sample(w, sample_rows, Z_sample, aop)
    return out


def run_epoch(workload: str, steps: int, warmup: int, with_cpu: bool):
    """Secondary workloads e1 / e2: one step = one minibatch embedding epoch (fusedmm_minibatch_epoch):
    per batch of 256 vertices two FusedMM executes on a rectangular slice and one update of its rows."""
    import numpy as np
    import torch
    from paper_2011_06391_amd import binding, model, synth

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (torch.cuda.is_available() is False)")
    binding.load()
    w = synth.make_epoch_workload(workload)
    g, d = w.csr, w.d
    rp, ci = torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda()
    neg = torch.from_numpy(w.negatives).cuda()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    mb = binding.Minibatch(g.m, rp, ci, w.batch_rows, neg)
    mb.reserve(d)
    torch.cuda.synchronize()
    plan_ms = (time.perf_counter() - t0) * 1e3
    info = mb.info()
    X = torch.from_numpy(w.X0).cuda()
    for _ in range(warmup):
        mb.epoch(X, w.lr)
    X.copy_(torch.from_numpy(w.X0).cuda())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        mb.epoch(X, w.lr)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / steps
    assert torch.isfinite(X).all().item()
    entries = g.nnz + g.m * w.n_negative          # stored entries processed per epoch, both calls
    pos = model.traffic(g.m, g.n, g.nnz, d, True, False, True)
    negt = model.traffic(g.m, g.n, g.m * w.n_negative, d, True, False, True)
    alg_bytes = pos.model_bytes + negt.model_bytes + 4 * g.m * d * 4   # + the update: read Zpos, Zneg, X, write X
    achieved = alg_bytes / (ms_per_step * 1e-3) / 1e9
    context = {}
    try:   # the same epoch replayed from a HIP graph (launch overhead of the host removed)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            mb.epoch(X, w.lr)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        context["ms_per_epoch_hip_graph"] = (time.perf_counter() - t0) * 1e3 / steps
        del graph
    except Exception as exc:
        context["hip_graph_error"] = repr(exc)[:200]
    # parity of one epoch from the initial embedding (checked on the CPU leg)
    X.copy_(torch.from_numpy(w.X0).cuda())
    mb.epoch(X, w.lr)
    torch.cuda.synchronize()
    X1 = X.cpu().numpy()
    mb.close()
    out = {
        "metric": "fused SDDMM-SpMM throughput: G(edge*dim)/s + achieved HBM GB/s vs peak, 1 GPU",
        "value": entries * d / (ms_per_step * 1e-3) / 1e9, "unit": "G(edge*dim)/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload, "description": w.description, "step": "one minibatch embedding epoch",
                   "n": g.m, "nnz": g.nnz, "d": d, "batch_rows": w.batch_rows, "n_negative": w.n_negative,
                   "n_batches": info["n_batches"], "launches_per_epoch": info["launches_per_epoch"],
                   "entries_per_epoch": entries, "plan_ms": plan_ms, "context": context},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": model.MI355X_HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / model.MI355X_HBM_PEAK_GBS, "traffic": None,
                     "note": "whole epoch (all launches), not one kernel: launches of 256 rows are latency-bound",
                     "algorithmic_bytes": alg_bytes},
    }
    if with_cpu:
        import oracle
        t0 = time.perf_counter()
        Xr, S = oracle.embedding_epoch(g.rowptr, g.colidx, w.X0, w.batch_rows, w.negatives, w.lr)
        cpu_s = time.perf_counter() - t0
        bound = 1e-4 * S + 2.0 ** -22 * np.abs(Xr)
        excess = float((np.abs(X1.astype(np.float64) - Xr.astype(np.float64)) - bound).max())
        out["cpu_baseline"] = {"value": entries * d / cpu_s / 1e9, "unit": "G(edge*dim)/s",
                               "cores": synth.num_threads(), "kind": "oracle",
                               "sample": "one whole epoch of the same workload, fp64 two-phase oracle", "seconds": cpu_s,
                               "parity_of_one_epoch": {"max_excess_over_bound": excess, "ok": excess <= 0.0,
                                                       "rule": "|X_gpu - X_oracle| <= 1e-4 * lr * sum|terms| + 2^-22 |X|"}}
    return out


HEADLINE = "c5"            # the largest configuration that fits one GPU: the workload of the default line
OTHER_WORKLOADS = ("c2", "c3", "c4")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=None, help="c1..c5 (default c5, the largest single-GPU configuration; the default run also "
                         "reports c2, c3 and c4 under config.all_workloads); e1, e2: minibatch embedding epochs (secondary); "
                         "rmat:SCALE:PAIRS: an R-MAT graph of that size for density sweeps (secondary)")
    ap.add_argument("--all-workloads", action="store_true",
                    help="also measure c2, c3 and c4 and report them under config.all_workloads (on when --workload is not given)")
    ap.add_argument("--d", type=int, default=None, help="override the feature dimension")
    ap.add_argument("--natural-order", action="store_true",
                    help="keep the vertex labels as generated (hubs at low ids) instead of the seeded random permutation "
                         "(secondary column: the gathers are then flattered by locality)")
    ap.add_argument("--aop", default="SUM", choices=("SUM", "MAX", "MIN", "MEAN"),
                    help="pool the workload's messages this way instead of summing them (secondary measurements)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the context measurements after the timed region (HIP-graph replay, copy bandwidth, "
                         "gather ceiling, cold caches), so that a profiler sees the benchmark launches only")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also launch the plain copy kernel once over this many MiB (profiler calibration)")
    ap.add_argument("--small-row-max", type=int, default=0)
    ap.add_argument("--split-row-min", type=int, default=0)
    ap.add_argument("--chunk-edges", type=int, default=0)
    ap.add_argument("--autotune", action="store_true", help="choose the schedule with fusedmm_plan_create_tuned")
    ap.add_argument("--y-f16", action="store_true",
                    help="optional storage mode: gather Y from an IEEE half copy (not the headline configuration)")
    ap.add_argument("--y-bf16", action="store_true",
                    help="optional storage mode: gather Y from a bfloat16 copy (not the headline configuration)")
    ap.add_argument("--f64", action="store_true",
                    help="the whole step in double precision through fusedmm_execute_f64 (not the headline configuration)")
    ap.add_argument("--column-classes", type=int, default=0)
    ap.add_argument("--tile-row-min", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        raise SystemExit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    workload = (args.workload or HEADLINE).lower()
    if workload in ("e1", "e2"):
        steps = args.steps if args.steps != 100 else 50
        warmup = args.warmup if args.warmup != 20 else 5
        print(json.dumps(run_epoch(workload, steps, warmup, not args.no_cpu_baseline)))
        return
    options = None
    if args.small_row_max or args.split_row_min or args.chunk_edges or args.column_classes or args.tile_row_min:
        options = {"small_row_max": args.small_row_max, "split_row_min": args.split_row_min,
                   "chunk_edges": args.chunk_edges, "column_classes": args.column_classes,
                   "tile_row_min": args.tile_row_min}
    y_storage = "f64" if args.f64 else ("bf16" if args.y_bf16 else ("f16" if args.y_f16 else "f32"))
    out = run(workload, args.steps, args.warmup, not args.no_cpu_baseline, options, args.d,
              args.copy_calibration_mib, args.autotune, y_storage, not args.no_context, not args.natural_order,
              aop=args.aop)
    if args.all_workloads or args.workload is None:
        # the other large configurations, same protocol (the same K timed steps, default plan), shorter report
        others = {}
        for name in OTHER_WORKLOADS:
            if name == workload:
                continue
            try:
                o = run(name, args.steps, args.warmup, not args.no_cpu_baseline, None, None, 0, False, "f32", False,
                        not args.natural_order, time_cpu=False)
                r = o["roofline"]
                others[name] = {"value": o["value"], "ms_per_step": o["ms_per_step"], "kernel_ms": r["kernel_ms"],
                                "nnz": o["config"]["nnz"], "d": o["config"]["d"], "pattern": o["config"]["pattern"],
                                "roofline_frac": r["frac"], "roofline_achieved_basis": r["achieved_basis"],
                                "traffic": r["traffic"], "l2_hit_rate": r["l2_hit_rate"],
                                "algorithmic_over_peak": r["algorithmic_over_peak"],
                                "parity_of_timed_result": o.get("cpu_baseline", {}).get("parity_of_timed_result")}
            except Exception as exc:   # secondary figures never break the headline line
                others[name] = {"error": repr(exc)[:300]}
        out["config"]["all_workloads"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
