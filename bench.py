#!/usr/bin/env python3
"""Throughput of the gradient-aggregation path on one MI355X.

A "step" is one whole iteration of the path over one batch of synthetic
gradients for all P simulated workers: fuse + accumulate + chunk norms + pack +
historical-gradient rule (gf_fuse_pack), ring reduce (gf_ring_reduce_sim),
unpack (gf_unpack_apply) and scoring / selection for the next iteration
(gf_chunk_score_select).  All inputs are resident in HBM before the timed
region.  The metric is algorithmic bytes per step / time per step (GB/s) and
its share of the 8 TB/s HBM peak.

Prints ONE JSON line.  `roofline` describes the dominant kernel, timed with
events on the launch stream inside the timed region; `cpu_baseline` is the CPU
checker run on the host cores on a bounded sample of the same workload.
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

# HBM traffic per launch of the dominant kernel measured with rocprofv3 --pmc
# (FETCH_SIZE and WRITE_SIZE runs, scaled by a copy kernel of known size); see
# profiles/.  Keyed by workload; absent -> null in the JSON.
MEASURED_TRAFFIC_BYTES = {
    # k_fuse<MODE_FUSED>: FETCH 3 820 996.6 x 2.0000 KiB + WRITE 4 002 746.6 x 1.0000 KiB per launch
    # (profiles/k_fuse_fused_alexnet_csc.md); counted between L2 and the fabric
    "alexnet_csc": 7825400947 + 4098812480,
}


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
    if sgd:                                   # Algorithm 1's update step: hu and w read and written
        st["unpack"] += L * 16
    return sum(st.values()), st


def run_gpu(name: str, steps: int, warmup: int, mode: str, schedule: str, n_sets: int, chunk=None,
            all_stages: bool = False, sgd=None, graph: bool = False):
    import torch
    from paper_1902_06855_amd import gf, pipeline as pl, workloads as wl

    w = wl.config(name)
    if chunk:                      # tuning aid: same tensors, another chunk size
        w.chunk = int(chunk)
    if os.environ.get("GF_BENCH_P"):   # tuning aid: another worker count
        w.P = int(os.environ["GF_BENCH_P"])
    torch.cuda.set_device(0)
    sig = wl.sigma_table(w)
    pipe_k = 0
    probe_plan = gf.Plan(w.sizes, min(w.theta, 1 << 60), w.chunk, w.P, to_device=False)
    if w.chunk:
        pipe_k = w.k_for(probe_plan.n_chunks)
    off, _, _ = probe_plan.layout()
    probe_plan.close()
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=pipe_k, mu=w.mu, wire=w.wire,
                       schedule=schedule, sgd=sgd, grad=w.grad, zero_copy=bool(w.extra.get("zero_copy")),
                       groups=int(w.extra.get("groups", 0)))
    if w.extra.get("zero_copy"):
        mode = "pool"
    # gradient sets resident in HBM: scattered per-tensor allocations (fusion is folded into the
    # read) or one pool per worker (the zero-copy layout)
    tables, keep = [], []
    t_gen = time.perf_counter()
    for s in range(n_sets):
        if mode == "gather":
            g = wl.gradients(w, s, device="cuda", sig=sig)
            keep.append(g)
            tables.append((gf.ptr_table([t for row in g for t in row]), None))
        else:
            pools = []
            for p in range(w.P):
                pool = torch.empty(w.N, dtype=torch.float16 if w.grad == "f16" else torch.float32, device="cuda")
                for l in range(w.m):
                    pool[off[l]:off[l] + w.sizes[l]] = wl.gradient_tensor(w, sig, s, p, l, "cuda")
                pools.append(pool)
            keep.append(pools)
            tables.append((None, gf.ptr_table(pools)))
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    it = 0
    for _ in range(warmup):
        pipe.use_tables(*tables[it % n_sets]); pipe.step(); it += 1
    torch.cuda.synchronize()
    _, st_bytes = algorithmic_bytes(w, pipe.cap, schedule, sgd is not None)
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
        # events bracket only the dominant kernel unless a per-stage breakdown is asked for: every
        # event is a packet between two kernels and costs a few microseconds of the step
        pipe.probe, pipe.probe_only = [], (None if all_stages else max(st_bytes, key=st_bytes.get))
        t0 = time.perf_counter()
        for _ in range(steps):
            pipe.use_tables(*tables[it % n_sets]); pipe.step(); it += 1
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        probe, pipe.probe = pipe.probe, None

    ms_per_step = (t1 - t0) * 1e3 / steps
    L = int(pipe.packed_len.item()) if w.chunk else w.N
    total_bytes, per_stage_bytes = algorithmic_bytes(w, L, schedule, sgd is not None)
    stage_ms = {}
    for nm, e0, e1 in probe:
        stage_ms.setdefault(nm, []).append(e0.elapsed_time(e1))
    stage_avg = {nm: sum(v) / len(v) for nm, v in stage_ms.items()}
    dominant = max(per_stage_bytes, key=per_stage_bytes.get)
    res = {
        "workload": name, "P": w.P, "N": w.N, "m": w.m, "chunk": w.chunk, "k": pipe_k, "L": L,
        "schedule": schedule if w.chunk else "dense", "input": mode, "n_buckets": pipe.plan.n_buckets,
        "ms_per_step": ms_per_step, "bytes_per_step": total_bytes,
        "gbs": total_bytes / ms_per_step / 1e6, "payload_gbs": w.P * w.N * (2 if w.grad == "f16" else 4) / ms_per_step / 1e6,
        "elements_per_s": w.P * w.N / ms_per_step * 1e3,
        "stage_ms": stage_avg, "stage_bytes": per_stage_bytes, "dominant": dominant,
        "dominant_ms": stage_avg.get(dominant), "gen_s": t_gen, "steps_timed": steps,
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


def stream_probe():
    """What bare kernels of the same access mixes sustain on this GPU (a stand-alone executable
    that shares nothing with the library): context for the roofline fraction.  None if absent."""
    import json as _json
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_1902_06855_amd", "probe", "stream_probe.bin")
    if not os.path.exists(exe):
        return None
    try:
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
        return _json.loads(r.stdout.strip().splitlines()[-1]) if r.returncode == 0 else None
    except Exception:
        return None


def cpu_baseline(name: str, schedule: str, threads: int):
    """The CPU checker, as it stands, on host cores: one whole steady-state iteration of the same
    workload with the worker count cut down so that the run stays bounded.  Timed twice on the
    same inputs: with `threads` OpenMP threads (the reported value) and with one."""
    import numpy as np
    from oracle import binding as ob, pipeline as op
    from paper_1902_06855_amd import workloads as wl

    w = wl.config(name)
    P_s = min(w.P, 8)                      # sample: the first P_s workers, every tensor, full size
    ws = wl.Workload(w.name + "_sample", w.sizes, P_s, w.chunk, w.density, w.loss_scale, w.theta,
                     w.iterations, w.mu, w.seed, w.wire)
    sig = wl.sigma_table(w)[:, :P_s]
    pools = []
    for t in range(2):
        g = [[wl.gradient_tensor(w, sig, t, p, l, "cpu").numpy() for l in range(w.m)] for p in range(P_s)]
        pools.append(np.stack([op.fuse(row, w.sizes) for row in g]))
        del g

    TIMED = 3                              # steady-state iterations per timing, averaged

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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="alexnet_csc")
    ap.add_argument("--input", choices=["gather", "pool"], default="gather")
    ap.add_argument("--schedule", choices=["lagged", "immediate"], default="lagged")
    ap.add_argument("--others", default="alexnet_dense,resnet50_dense_4mb,resnet50_dense_64mb,resnet50_csc",
                    help="comma-separated extra workloads reported under config.others ('' = none)")
    ap.add_argument("--ladder", action="store_true",
                    help="also report the lower rungs of the ladder of Tables 1-2 (per-tensor fp32 / fp16 "
                         "allreduce) and the fp16-input variants under config.others")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage-times", action="store_true", help="bracket every stage with events (adds a few us per step)")
    ap.add_argument("--chunk", type=int, default=None, help="override the workload's chunk size (tuning aid)")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: first a plain elementwise copy of known size (2 GiB read, "
                         "2 GiB written) that calibrates the byte counters, then a short run of the workload")
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
    steps = a.steps if a.steps is not None else max(10, w.iterations)
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
    main_res = run_gpu(a.workload, steps, warmup, a.input, a.schedule, n_sets, a.chunk, a.stage_times)
    others = {}
    for nm in [x for x in a.others.split(",") if x and x != a.workload]:
        wo = wl.config(nm)
        so = max(10, wo.iterations)
        r = run_gpu(nm, so, 5, a.input, a.schedule, min(so, 10) if wo.chunk else 2, None, a.stage_times)
        others[nm] = {kk: r[kk] for kk in ("P", "N", "schedule", "n_buckets", "ms_per_step", "gbs", "payload_gbs",
                                            "stage_ms", "dominant", "dominant_ms")}
        others[nm]["frac_of_hbm_peak"] = r["gbs"] / HBM_PEAK_GBS
        dom_b = r["stage_bytes"][r["dominant"]]
        others[nm]["dominant_gbs"] = dom_b / r["dominant_ms"] / 1e6

    if not a.pmc_probe and a.others:
        # the same iterations replayed as HIP graphs (no events inside: whole-iteration time only)
        for nm in [a.workload] + [x for x in a.others.split(",") if x and x != a.workload and "dense" in x][:2]:
            wo = wl.config(nm)
            so = max(10, wo.iterations)
            r = run_gpu(nm, so, 5, a.input, a.schedule, min(so, 10) if wo.chunk else 2, None, False, None, True)
            others[nm + "+graph"] = {kk: r[kk] for kk in ("P", "N", "schedule", "ms_per_step", "gbs", "bytes_per_step")}
            others[nm + "+graph"]["frac_of_hbm_peak"] = r["gbs"] / HBM_PEAK_GBS
    if a.ladder and not a.pmc_probe:
        for nm in ("alexnet_dense", "resnet50_dense_4mb", "resnet50_pertensor_fp16"):
            others[nm + "+buckets_on_side_streams"] = run_overlap(nm, 10, 5, 4)
    if w.chunk and not a.pmc_probe and a.others:
        # the same workload with Algorithm 1's SGD-update step fused into the unpack
        r = run_gpu(a.workload, steps, warmup, a.input, a.schedule, n_sets, a.chunk, a.stage_times, (0.9, -0.01))
        others[a.workload + "+sgd_update"] = {kk: r[kk] for kk in ("P", "N", "schedule", "ms_per_step", "gbs",
                                                                      "bytes_per_step", "stage_ms")}
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
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32->f16" if w.wire == "f16" else "f32", "data": "synthetic",
        "frac_of_hbm_peak": main_res["gbs"] / HBM_PEAK_GBS,
        "payload_gbs": main_res["payload_gbs"], "elements_per_s": main_res["elements_per_s"],
        "config": {"workload": a.workload, "P": w.P, "N": w.N, "tensors": w.m, "chunk": w.chunk,
                   "k": main_res["k"], "packed_elems": main_res["L"], "loss_scale": w.loss_scale,
                   "schedule": main_res["schedule"], "input": a.input,
                   "bytes_per_step": main_res["bytes_per_step"], "stage_ms": main_res["stage_ms"],
                   "gradient_sets_resident": n_sets, "others": others},
        "roofline": {"bound": "hbm", "kernel": kernel, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "bytes_per_launch": dom_bytes,
                     "avg_launch_ms": main_res["dominant_ms"],
                     "traffic": MEASURED_TRAFFIC_BYTES.get(a.workload)},
    }
    if not a.pmc_probe:
        # a child process, run after the timed work (5 GB of its own buffers)
        out["roofline"]["bare_kernel_reference"] = stream_probe()
    if not a.no_cpu_baseline:
        ncpu = min(16, os.cpu_count() or 1)
        out["cpu_baseline"] = cpu_baseline(a.workload, a.schedule, ncpu)
        out["cpu_baseline"]["gpu_over_cpu"] = main_res["gbs"] / out["cpu_baseline"]["value"]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
