#!/usr/bin/env python3
"""Throughput of the gradient-aggregation path on one MI355X.

A "step" is one whole iteration of the path over one batch of synthetic
gradients for all P simulated workers: fuse + accumulate + chunk norms + pack +
historical-gradient rule (gf_fuse_pack), ring reduce (gf_ring_reduce_sim),
unpack (gf_unpack_apply) and scoring / selection for the next iteration
(gf_chunk_score_select).  All inputs are resident in HBM before the timed
region.  The metric is algorithmic bytes per step / time per step (GB/s) and
its share of the 8 TB/s HBM peak.

Prints ONE JSON line.  `value` comes from the wall clock around exactly K steps
(synchronised on both sides); `median_ms` / `min_ms` from one event per
iteration boundary on the launch stream; `roofline` describes the dominant
kernel, bracketed by events on the launch stream inside the timed region;
`config.stages` gives every stage's time and GB/s from a second, untimed pass
with every stage bracketed; `cpu_baseline` is the CPU checker run on the host
cores on a bounded sample of the same workload.  `config.others` holds the
other configurations, one-worker rows (the shape one GPU of a real job runs),
the same iterations replayed as HIP graphs (`+graph`), issued by one host call
each (`+one_call`, gf_csc_iteration) and with Algorithm 1's update step fused
into the unpack (`+sgd_update`); `--ladder` adds the lower rungs of Tables 1-2.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic per launch of the dominant kernel measured with rocprofv3 --pmc (one FETCH_SIZE run,
# one WRITE_SIZE run, each scaled by what the same counter reads for a copy of known size): bytes
# read + bytes written between L2 and the fabric, from the tables under profiles/.  Keyed by
# (workload, input layout, schedule): a run in any other configuration reports null.
MEASURED_TRAFFIC_BYTES = {
    # profiles/k_fuse_fused_resnet50_csc.md: FETCH 6 394 802.1 x 2 KiB + WRITE 6 423 586.2 KiB per launch
    ("resnet50_csc", "gather", "lagged"): 13096554688 + 6577752272,
    # profiles/k_fuse_fused_alexnet_csc.md: FETCH 3 813 246.4 x 2 KiB + WRITE 4 002 746.6 KiB per launch
    ("alexnet_csc", "gather", "lagged"): 7809528704 + 4098812552,
    # profiles/kernel_stats_other_workloads.md, cast kernel: FETCH 953 915.5 x 2 KiB + WRITE 952 581.8 KiB
    ("alexnet_dense", "gather", "dense"): 1953619021 + 975443712,
}

DEFAULT_WORKLOAD = "resnet50_csc"     # the largest single-GPU configuration of the five
DEFAULT_OTHERS = "alexnet_csc,alexnet_dense,resnet50_dense_4mb,resnet50_dense_64mb,resnet50_csc_p1,alexnet_csc_p1"


def algorithmic_bytes(w, k_elems_L: int, schedule: str, sgd: bool = False):
    """Bytes the method must move per iteration (every gradient read once, the
    historical gradient read and written once, each wire element written once
    and read once per worker, the reduced buffer written once and read once,
    each output written once).  Returns (total, per-stage dict)."""
    P, N, L = w.P, w.N, k_elems_L
    ws = 2 if w.wire == "f16" else 4
    gs = 2 if w.grad == "f16" else 4          # bytes per gradient element as it arrives
    if w.chunk == 0 and w.extra.get("zero_copy"):
        st = {"ring": N * (P * ws + ws), "unpack": N * (ws + 4)}
    elif w.chunk == 0:
        st = {"cast": P * N * (gs + ws), "ring": N * (P * ws + ws), "unpack": N * (ws + 4)}
    elif schedule == "lagged":
        st = {"fused": P * N * (gs + 8) + P * L * ws, "ring": L * (P * ws + ws), "unpack": L * (ws + 4), "select": 0}
    else:
        st = {"accum": P * N * (gs + 8), "pack": P * L * (4 + ws + 4), "ring": L * (P * ws + ws),
              "unpack": L * (ws + 4), "select": 0}
    if sgd:                                   # Algorithm 1's update step: hu and w read and written,
        st["unpack"] += L * 18                #   the FP16 copy of the updated weights written (Section 2.5)
    return sum(st.values()), st


def resident_gradient_sets(w, n_sets: int, mode: str, few_dispatches: bool = False):
    """n_sets gradient sets resident in HBM and their pointer tables: scattered per-tensor
    allocations (mode "gather": fusion is folded into the read) or one pool per worker (mode
    "pool": the zero-copy layout).  few_dispatches draws each worker's set with one generator
    launch (the tensors are then slices of one allocation, still reached through the per-tensor
    pointer table): for runs under a counter-collecting profiler, which must not see the tens of
    thousands of small launches of the per-tensor generator."""
    import torch
    from paper_1902_06855_amd import gf, workloads as wl

    sig = wl.sigma_table(w)
    plan = gf.Plan(w.sizes, min(w.theta, 1 << 60), w.chunk, w.P, to_device=False)
    off, _, _ = plan.layout()
    plan.close()
    gdt = torch.float16 if w.grad == "f16" else torch.float32
    tables, keep = [], []
    for s in range(n_sets):
        if few_dispatches:
            pools = []
            for p in range(w.P):
                g = torch.Generator(device="cuda")
                g.manual_seed(wl.stream_seed(w.seed, s, p, 0xFEED))
                x = torch.randn(w.N, generator=g, device="cuda", dtype=torch.float32)
                x.mul_(float(sig[:, p].mean()))
                pools.append(x.to(gdt))
            keep.append(pools)
            if mode == "gather":
                tables.append((gf.ptr_table([pools[p][off[l]:off[l] + w.sizes[l]] for p in range(w.P)
                                             for l in range(w.m)]), None))
            else:
                tables.append((None, gf.ptr_table(pools)))
        elif mode == "gather":
            g = wl.gradients(w, s, device="cuda", sig=sig)
            keep.append(g)
            tables.append((gf.ptr_table([t for row in g for t in row]), None))
        else:
            pools = []
            for p in range(w.P):
                pool = torch.empty(w.N, dtype=gdt, device="cuda")
                for l in range(w.m):
                    pool[off[l]:off[l] + w.sizes[l]] = wl.gradient_tensor(w, sig, s, p, l, "cuda")
                pools.append(pool)
            keep.append(pools)
            tables.append((None, gf.ptr_table(pools)))
    torch.cuda.synchronize()
    return tables, keep


def run_gpu(name: str, steps: int, warmup: int, mode: str, schedule: str, n_sets: int,
            sgd=None, graph: bool = False, few_dispatches: bool = False, stage_pass: bool = True,
            one_call: bool = False):
    import torch
    from paper_1902_06855_amd import gf, pipeline as pl, workloads as wl

    w = wl.config(name)
    torch.cuda.set_device(0)
    pipe_k = 0
    if w.chunk:
        probe_plan = gf.Plan(w.sizes, min(w.theta, 1 << 60), w.chunk, w.P, to_device=False)
        pipe_k = w.k_for(probe_plan.n_chunks)
        probe_plan.close()
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=pipe_k, mu=w.mu, wire=w.wire,
                       schedule=schedule, sgd=sgd, half_weights=sgd is not None, grad=w.grad,
                       zero_copy=bool(w.extra.get("zero_copy")),
                       groups=int(w.extra.get("groups", 0)))
    if w.extra.get("zero_copy"):
        mode = "pool"
    t_gen = time.perf_counter()
    tables, keep = resident_gradient_sets(w, n_sets, mode, few_dispatches)
    t_gen = time.perf_counter() - t_gen

    it = 0
    for _ in range(warmup):
        pipe.use_tables(*tables[it % n_sets]); pipe.step(); it += 1
    torch.cuda.synchronize()
    _, st_bytes = algorithmic_bytes(w, pipe.cap, schedule, sgd is not None)
    dominant = max(st_bytes, key=st_bytes.get)
    iter_ms = []
    if graph:
        # every iteration replayed as one HIP graph (one graph per resident gradient set: the
        # tables are baked in); no events inside a graph, so no per-kernel times in this mode
        graphs = []
        for s in range(n_sets):
            pipe.use_tables(*tables[s]); graphs.append(pipe.capture())
        for s in range(n_sets):
            graphs[s].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graphs[it % n_sets].replay(); it += 1
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        probe = []
    else:
        # inside the timed region: one event per iteration boundary, and events around the dominant
        # stage only (every event is a packet between two kernels and costs a few microseconds)
        # (one_call: no events inside the iteration at all, so that a steady-state sparse iteration
        # is the library's single gf_csc_iteration call)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        if not one_call:
            pipe.probe, pipe.probe_only = [], dominant
        t0 = time.perf_counter()
        for i in range(steps):
            marks[i].record()
            pipe.use_tables(*tables[it % n_sets]); pipe.step(); it += 1
        marks[steps].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        probe, pipe.probe = pipe.probe or [], None
        iter_ms = [marks[i].elapsed_time(marks[i + 1]) for i in range(steps)]

    ms_per_step = (t1 - t0) * 1e3 / steps
    L = int(pipe.packed_len.item()) if w.chunk else w.N
    total_bytes, per_stage_bytes = algorithmic_bytes(w, L, schedule, sgd is not None)
    dom_ms = [e0.elapsed_time(e1) for nm, e0, e1 in probe if nm == dominant]

    # second pass, outside the timed region: every stage bracketed
    stages = {}
    if stage_pass and not graph and not one_call:
        pipe.probe, pipe.probe_only = [], None
        for _ in range(min(steps, 10)):
            pipe.use_tables(*tables[it % n_sets]); pipe.step(); it += 1
        torch.cuda.synchronize()
        probe2, pipe.probe = pipe.probe, None
        per = {}
        for nm, e0, e1 in probe2:
            per.setdefault(nm, []).append(e0.elapsed_time(e1))
        for nm, v in per.items():
            med = statistics.median(v)
            b = per_stage_bytes.get(nm, 0)
            stages[nm] = {"median_ms": med, "min_ms": min(v), "bytes": b,
                          "gbs": (b / med / 1e6) if b else None}

    res = {
        "workload": name, "P": w.P, "N": w.N, "m": w.m, "chunk": w.chunk, "k": pipe_k, "L": L,
        "schedule": schedule if w.chunk else "dense", "input": mode, "n_buckets": pipe.plan.n_buckets,
        "ms_per_step": ms_per_step, "bytes_per_step": total_bytes,
        "median_ms": statistics.median(iter_ms) if iter_ms else None,
        "min_ms": min(iter_ms) if iter_ms else None,
        "gbs": total_bytes / ms_per_step / 1e6,
        "payload_gbs": w.P * w.N * (2 if w.grad == "f16" else 4) / ms_per_step / 1e6,
        "elements_per_s": w.P * w.N / ms_per_step * 1e3,
        "stage_bytes": per_stage_bytes, "dominant": dominant, "stages": stages,
        "dominant_ms": (sum(dom_ms) / len(dom_ms)) if dom_ms else None,
        "dominant_median_ms": statistics.median(dom_ms) if dom_ms else None,
        "dominant_min_ms": min(dom_ms) if dom_ms else None,
        "gen_s": t_gen, "steps_timed": steps,
    }
    del keep, tables, pipe
    torch.cuda.empty_cache()
    return res


def run_overlap(name: str, steps: int, warmup: int, n_streams: int = 2):
    """A dense workload with every lazy-allreduce bucket issued on its own (cast, ring, cast back)
    on side streams in generation order: the enable-overlap setting, with nothing to overlap
    with here, so this shows what issuing bucket by bucket costs."""
    import torch
    from paper_1902_06855_amd import pipeline as pl, workloads as wl

    w = wl.config(name)
    torch.cuda.set_device(0)
    sig = wl.sigma_table(w)
    ov = pl.OverlappedDense(w.sizes, w.P, w.theta, w.loss_scale, wire=w.wire, n_streams=n_streams)
    sets, tabs = [], []
    for s in range(2):
        g = wl.gradients(w, s, device="cuda", sig=sig)
        ov.set_gradients(g)
        sets.append(g); tabs.append(ov.grad_tabs)
    it = 0
    for _ in range(warmup):
        ov.grad_tabs = tabs[it % 2]; ov.step(); it += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ov.grad_tabs = tabs[it % 2]; ov.step(); it += 1
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    total, _ = algorithmic_bytes(w, w.N, "dense")
    # the same, each iteration replayed as one HIP graph (no host launches in the timed region)
    graphs = []
    for s in range(2):
        ov.grad_tabs = tabs[s]; graphs.append(ov.capture())
    for s in range(2):
        graphs[s].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graphs[it % 2].replay(); it += 1
    torch.cuda.synchronize()
    ms_graph = (time.perf_counter() - t0) * 1e3 / steps
    res = {"P": w.P, "N": w.N, "n_buckets": ov.n_buckets, "streams": n_streams, "ms_per_step": ms,
           "gbs": total / ms / 1e6, "bytes_per_step": total, "frac_of_hbm_peak": total / ms / 1e6 / HBM_PEAK_GBS,
           "ms_per_step_as_graph": ms_graph, "gbs_as_graph": total / ms_graph / 1e6}
    del ov, sets, tabs
    torch.cuda.empty_cache()
    return res


def run_overlap_csc(name: str, steps: int, warmup: int, n_ranges: int = 8, buckets: int = 4):
    """A sparse workload swept range by range (n_ranges equal chunk ranges in generation order) with
    the packed buffer reduced and unpacked bucket by bucket (theta = a quarter of it) on a second
    stream while the next ranges are swept: Section 3.2's enable-overlap setting, with no backward
    to overlap with here, so this shows what issuing range by range costs against the single pass."""
    import torch
    from paper_1902_06855_amd import gf, pipeline as pl, workloads as wl

    w = wl.config(name)
    torch.cuda.set_device(0)
    plan = gf.Plan(w.sizes, 1 << 60, w.chunk, w.P, to_device=False)
    nc = plan.n_chunks
    plan.close()
    k = w.k_for(nc)
    theta = max(1, k // buckets) * w.chunk - 1          # a bucket closes every k / buckets packed chunks
    bounds = sorted({max(1, (r + 1) * nc // n_ranges) for r in range(n_ranges)} | {nc})
    ov = pl.OverlappedCsc(w.sizes, w.P, w.chunk, theta, w.loss_scale, k, bounds, mu=w.mu, wire=w.wire)
    n_sets = 3
    tables, keep = resident_gradient_sets(w, n_sets, "gather")
    it = 0
    for _ in range(warmup):
        ov.pipe.use_tables(*tables[it % n_sets]); ov.step(); it += 1
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ov.pipe.use_tables(*tables[it % n_sets]); ov.step(); it += 1
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    L = int(ov.pipe.packed_len.item())
    total, _ = algorithmic_bytes(w, L, "lagged")
    graphs = []
    for s in range(n_sets):                              # one recorded iteration per resident gradient set
        ov.pipe.use_tables(*tables[s]); graphs.append(ov.capture())
    for s in range(n_sets):
        graphs[s].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graphs[it % n_sets].replay(); it += 1
    torch.cuda.synchronize()
    ms_graph = (time.perf_counter() - t0) * 1e3 / steps
    res = {"P": w.P, "N": w.N, "chunk_ranges": len(bounds), "packed_buckets": -(-k // max(1, k // buckets)),
           "ms_per_step": ms, "gbs": total / ms / 1e6, "bytes_per_step": total,
           "frac_of_hbm_peak": total / ms / 1e6 / HBM_PEAK_GBS,
           "ms_per_step_as_graph": ms_graph, "gbs_as_graph": total / ms_graph / 1e6}
    del ov, tables, keep
    torch.cuda.empty_cache()
    return res


def cpu_baseline(name: str, schedule: str, threads: int):
    """The CPU checker, as it stands, on host cores: whole steady-state iterations of the same
    workload with the worker count cut down so that the run stays bounded.  Timed twice on the
    same inputs: with `threads` OpenMP threads (the reported value) and with one."""
    import numpy as np
    from oracle import binding as ob, pipeline as op
    from paper_1902_06855_amd import workloads as wl

    w = wl.config(name)
    P_s = min(w.P, 16)                     # sample: the first P_s workers, every tensor, full size
    ws = wl.Workload(w.name + "_sample", w.sizes, P_s, w.chunk, w.density, w.loss_scale, w.theta,
                     w.iterations, w.mu, w.seed, w.wire)
    sig = wl.sigma_table(w)[:, :P_s]
    pools = []
    for t in range(2):
        g = [[wl.gradient_tensor(w, sig, t, p, l, "cpu").numpy() for l in range(w.m)] for p in range(P_s)]
        pools.append(np.stack([op.fuse(row, w.sizes) for row in g]))
        del g

    TIMED = 5                              # steady-state iterations per timing, averaged

    def once(nthreads):
        ob.set_threads(nthreads)
        used = ob.get_threads()
        if w.chunk:
            k = w.k_for(ob.n_chunks(w.N, w.chunk))
            state = op.new_state(P_s, w.N)
            op.csc_iteration(state, pools[0], w.chunk, k, w.loss_scale, w.mu, schedule, w.wire)   # iteration 0
            t0 = time.perf_counter()
            for t in range(TIMED):
                r = op.csc_iteration(state, pools[(t + 1) % 2], w.chunk, k, w.loss_scale, w.mu, schedule, w.wire)
            dt = (time.perf_counter() - t0) / TIMED
            L = r["send"].shape[1]
        else:
            t0 = time.perf_counter()
            for t in range(TIMED):
                op.dense_iteration(pools[(t + 1) % 2], w.sizes, w.theta, w.loss_scale, w.wire)
            dt = (time.perf_counter() - t0) / TIMED
            L = w.N
        total_bytes, _ = algorithmic_bytes(ws, L, schedule)
        return used, dt, total_bytes

    used, dt, total_bytes = once(threads)
    _, dt1, _ = once(1)
    return {
        "value": total_bytes / dt / 1e9, "unit": "GB/s", "cores": used, "kind": "oracle",
        "sample": f"{TIMED} steady-state {schedule if w.chunk else 'dense'} iterations of {name} with the first "
                  f"{P_s} of {w.P} workers (all {w.m} tensors, full size; bytes counted for {P_s} workers; "
                  f"seconds are per iteration)",
        "seconds": dt, "elements_per_s": P_s * w.N / dt,
        "single_thread_value": total_bytes / dt1 / 1e9, "single_thread_seconds": dt1,
    }


OTHER_KEYS = ("P", "N", "chunk", "k", "schedule", "n_buckets", "ms_per_step", "median_ms", "min_ms", "gbs",
              "payload_gbs", "bytes_per_step", "stages", "dominant", "dominant_ms")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--input", choices=["gather", "pool"], default="gather")
    ap.add_argument("--schedule", choices=["lagged", "immediate"], default="lagged")
    ap.add_argument("--others", default=DEFAULT_OTHERS,
                    help="comma-separated extra workloads reported under config.others ('' = none)")
    ap.add_argument("--ladder", action="store_true",
                    help="also report the lower rungs of the ladder of Tables 1-2 (per-tensor fp32 / fp16 "
                         "allreduce), the fp16-input, hierarchical-order, short-chunk and bucket-wise variants "
                         "under config.others")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for the rocprofv3 --pmc commands recorded under profiles/: first a plain elementwise "
                         "copy of known size (2 GiB read, 2 GiB written) that calibrates the byte counters, then 2 + 3 "
                         "iterations of the workload on gradient sets drawn with one generator launch per worker")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the P workers are simulated in one GPU's HBM); "
              "--gpus must be 1", file=sys.stderr)
        return 2
    if int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: launched with WORLD_SIZE > 1; this build has no multi-GPU path", file=sys.stderr)
        return 2
    from paper_1902_06855_amd import workloads as wl
    if a.ladder:
        a.others = ",".join([a.others] + list(wl.LADDER_NAMES))
    w = wl.config(a.workload)
    steps = a.steps if a.steps is not None else max(20, w.iterations)
    warmup = a.warmup if a.warmup is not None else 5
    n_sets = min(steps, 10) if w.chunk else 2

    if a.pmc_probe:
        import torch
        n = 1 << 29
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)       # reads 4n bytes, writes 4n bytes
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
        a.others, a.no_cpu_baseline = "", True
        steps, warmup, n_sets = 3, 2, 2
    main_res = run_gpu(a.workload, steps, warmup, a.input, a.schedule, n_sets,
                       few_dispatches=a.pmc_probe, stage_pass=not a.pmc_probe)
    others = {}
    for nm in [x for x in a.others.split(",") if x and x != a.workload]:
        wo = wl.config(nm)
        so = max(20, wo.iterations)
        r = run_gpu(nm, so, 5, a.input, a.schedule, min(so, 10) if wo.chunk else 2)
        others[nm] = {kk: r[kk] for kk in OTHER_KEYS}
        others[nm]["frac_of_hbm_peak"] = r["gbs"] / HBM_PEAK_GBS
        dom_b = r["stage_bytes"][r["dominant"]]
        others[nm]["dominant_gbs"] = dom_b / r["dominant_ms"] / 1e6

    if not a.pmc_probe and a.others:
        # the same iterations replayed as HIP graphs (no events inside: whole-iteration time only)
        named = [x for x in a.others.split(",") if x and x != a.workload]
        for nm in ([a.workload] + [x for x in named if "dense" in x][:2]
                   + [x for x in named if x.endswith("_p1") or x.endswith("_fp16pool")]):
            wo = wl.config(nm)
            so = max(20, wo.iterations)
            r = run_gpu(nm, so, 5, a.input, a.schedule, min(so, 10) if wo.chunk else 2, graph=True)
            others[nm + "+graph"] = {kk: r[kk] for kk in ("P", "N", "schedule", "ms_per_step", "gbs", "bytes_per_step")}
            others[nm + "+graph"]["frac_of_hbm_peak"] = r["gbs"] / HBM_PEAK_GBS
    if not a.pmc_probe and a.others:
        # sparse iterations issued by one host call each (gf_csc_iteration), no events inside
        named = [x for x in a.others.split(",") if x and x != a.workload]
        for nm in [a.workload] + [x for x in named if x.endswith("_csc_p1")]:
            wo = wl.config(nm)
            if not wo.chunk:
                continue
            so = max(20, wo.iterations)
            r = run_gpu(nm, so, 5, a.input, a.schedule, min(so, 10), one_call=True)
            others[nm + "+one_call"] = {kk: r[kk] for kk in ("P", "N", "schedule", "ms_per_step", "median_ms", "min_ms",
                                                             "gbs", "bytes_per_step")}
            others[nm + "+one_call"]["frac_of_hbm_peak"] = r["gbs"] / HBM_PEAK_GBS
    if a.ladder and not a.pmc_probe:
        for nm in ("alexnet_dense", "resnet50_dense_4mb", "resnet50_pertensor_fp16"):
            others[nm + "+buckets_on_side_streams"] = run_overlap(nm, 10, 5, 4)
        for nm in ("alexnet_csc", "resnet50_csc"):
            others[nm + "+ranges_and_buckets_as_they_fill"] = run_overlap_csc(nm, 10, 5)
    if w.chunk and not a.pmc_probe and a.others:
        # the same workload with Algorithm 1's SGD-update step (and the FP16 weight copy) fused into the unpack
        r = run_gpu(a.workload, steps, warmup, a.input, a.schedule, n_sets, sgd=(0.9, -0.01))
        others[a.workload + "+sgd_update"] = {kk: r[kk] for kk in ("P", "N", "schedule", "ms_per_step", "gbs",
                                                                      "bytes_per_step", "stages")}
        others[a.workload + "+sgd_update"]["frac_of_hbm_peak"] = r["gbs"] / HBM_PEAK_GBS
    dom = main_res["dominant"]
    dom_bytes = main_res["stage_bytes"][dom]
    achieved = dom_bytes / main_res["dominant_ms"] / 1e6
    kernel = {"fused": "k_fuse<MODE_FUSED> (gf_fuse_pack, accumulate+norms+pack+historical gradient)",
              "cast": "k_fuse<MODE_DENSE> (gf_fuse_pack, fused gather + scale + fp16 cast)",
              "accum": "k_fuse<MODE_ACCUM> (gf_fuse_pack, accumulate + norms)"}.get(dom, dom)
    out = {
        "metric": "gradient GB/s per step (fuse+sparsify+reduce) and % of MI355X HBM peak",
        "value": main_res["gbs"], "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": main_res["ms_per_step"], "median_ms": main_res["median_ms"], "min_ms": main_res["min_ms"],
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32->f16" if w.wire == "f16" else "f32", "data": "synthetic",
        "frac_of_hbm_peak": main_res["gbs"] / HBM_PEAK_GBS,
        "payload_gbs": main_res["payload_gbs"], "elements_per_s": main_res["elements_per_s"],
        "config": {"workload": a.workload, "P": w.P, "N": w.N, "tensors": w.m, "chunk": w.chunk,
                   "k": main_res["k"], "packed_elems": main_res["L"], "loss_scale": w.loss_scale,
                   "schedule": main_res["schedule"], "input": a.input,
                   "bytes_per_step": main_res["bytes_per_step"], "stages": main_res["stages"],
                   "gradient_sets_resident": n_sets, "others": others},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "bytes_per_launch": dom_bytes,
                     "avg_launch_ms": main_res["dominant_ms"], "median_launch_ms": main_res["dominant_median_ms"],
                     "min_launch_ms": main_res["dominant_min_ms"],
                     "traffic": MEASURED_TRAFFIC_BYTES.get((a.workload, a.input, main_res["schedule"]))},
    }
    if not a.no_cpu_baseline:
        ncpu = min(16, os.cpu_count() or 1)
        out["cpu_baseline"] = cpu_baseline(a.workload, a.schedule, ncpu)
        out["cpu_baseline"]["gpu_over_cpu"] = main_res["gbs"] / out["cpu_baseline"]["value"]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
