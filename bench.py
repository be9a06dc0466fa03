#!/usr/bin/env python3
"""Benchmark of the Dolphin hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N | --configs 1,2,3,4,5] [--batch B]

A step is one pass of a whole program (all its operator launches, forward and backward) over one batch of
seeded synthetic input already resident in HBM.  With no flags the five baseline workloads are measured one after
the other; the headline fields of the ONE JSON line printed (`value`, `ms_per_step`, `roofline`, `cpu_baseline`) are
those of workload 2, the Sum-15 DAMP chain forward + backward at B=4096, and `configs` holds one record per
workload: its step time, the roofline of its dominant kernel, the step against the bytes it must move at the very
least, the same program at a B-scaled batch, the CPU oracle timed on this host's cores, and the number of
clamp decisions that sit within 1e-6 of the clamp.

Clock: a timed region is `steps` steps issued `inner_repeats` times over, between two device synchronisations;
`inner_repeats` is raised until a region lasts at least --min-region-ms, and the step time is the median over
--regions regions.  Kernel times come from HIP events on the launch stream around back-to-back launches.
"""
from __future__ import annotations

import argparse
import datetime
import hashlib
import json
import math
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_PEAK_TFLOPS = 157.3       # MI355X fp32 vector, published: 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 flop x 2.4 GHz
FP32_NONPACKED_TFLOPS = 78.6   # the same without packed fp32 instructions, which this build does not use
SCALED_BATCH = {1: 1 << 22, 2: 1 << 19, 3: 1 << 18, 4: 1 << 18, 5: 1 << 13, 6: 1 << 11, 7: 1 << 11, 8: 1 << 12}
BASELINE_CONFIGS = (1, 2, 3, 4, 5)
NEAR_TIE = 1e-6


# ---------------------------------------------------------------------------------------------- timing

def make_runner(prog, torch, warmup, mode):
    """Untimed warmup; returns the callable that issues one step (the launches, or a HIP-graph replay of them)."""
    for _ in range(max(warmup, 1)):
        prog.step()
    torch.cuda.synchronize()
    if mode != "graph":
        return prog.step
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        prog.step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        prog.step()
    for _ in range(max(warmup, 1)):
        graph.replay()
    torch.cuda.synchronize()
    prog._graph = graph                     # keeps the graph alive as long as the program
    return graph.replay


def time_step(run, torch, steps, regions, min_region_ms):
    """Median over `regions` timed regions of the time of one step.  A region is steps * inner steps between two
    device synchronisations; inner is the smallest count that makes a region last min_region_ms."""
    def region(n):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n):
            run()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3
    probe = region(steps)
    inner = max(1, int(math.ceil(min_region_ms / max(probe, 1e-6))))
    inner = min(inner, 10000)
    ms = [region(steps * inner) for _ in range(regions)]
    per_step = [m / (steps * inner) for m in ms]
    return statistics.median(per_step), dict(regions=regions, steps_per_region=steps * inner, inner_repeats=inner,
                                             region_ms=[round(m, 3) for m in ms],
                                             ms_per_step_min=round(min(per_step), 6), ms_per_step_max=round(max(per_step), 6))


def copy_rate(torch, mib=1024, reps=5):
    """Read + write rate of a plain device-to-device copy of `mib` MiB (the runtime's copy kernel): what a streaming
    kernel reaches on this device, beside the published peak.  Also the known-size copy the traffic counters are
    calibrated with (--calibrate-copy)."""
    n = mib * (1 << 20) // 4
    src = torch.full((n,), 1.0, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    return round(2.0 * mib * (1 << 20) * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)


def time_launches(prog, torch, repeats, min_pair_ms=4.0):
    """Average duration of every launch of a step: back-to-back launches between two HIP events on the launch
    stream, as many as make the pair span min_pair_ms (at least `repeats`); the fastest of three such pairs.
    Returns {kernel: dict(launches, ms, bytes, macs)} summed over one step."""
    per_kernel = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def pair(l, n):
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            l.call()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)
    budget = min_pair_ms if len(prog.launches) <= 16 else min_pair_ms * 16 / len(prog.launches)
    for l in prog.launches:
        l.call()
        first = pair(l, repeats)
        n = max(repeats, int(math.ceil(repeats * budget / max(first, 1e-6))))
        ms = min(pair(l, n) for _ in range(3)) / n if n > repeats else first / repeats     # (the fastest of three pairs)
        k = per_kernel.setdefault(l.kernel, dict(launches=0, ms=0.0, bytes=0, macs=0))
        k["launches"] += 1
        k["ms"] += ms
        k["bytes"] += l.bytes
        k["macs"] += l.macs
    return per_kernel


# ---------------------------------------------------------------------------------------------- roofline

def _source_of(kernel):
    """The .hip file that defines `kernel`, and the sha256 of its text."""
    base = kernel.split("<")[0].strip()
    csrc = os.path.join(ROOT, "paper_2410_03348_amd", "csrc")
    for fn in sorted(os.listdir(csrc)):
        if fn.endswith(".hip"):
            text = open(os.path.join(csrc, fn)).read()
            if base + "(" in text:      # the definition, or the line that writes it for kernels generated at run time
                return fn, hashlib.sha256(text.encode()).hexdigest()[:16]
    return None, None


def measured_traffic(cfg, batch, kernel):
    """HBM bytes per launch of `kernel` on this workload as the profiler's FETCH_SIZE / WRITE_SIZE counters gave them:
    a table written from separate rocprofv3 --pmc runs (the counters cannot be read from inside this program).
    An entry counts only while the kernel's source file is the one that was profiled; otherwise the figure is
    withheld and the date of the stale profile returned instead."""
    path = os.path.join(ROOT, "paper_2410_03348_amd", "hbm_traffic.json")
    try:
        table = json.load(open(path))
        entries = table["entries"]
    except (OSError, ValueError, KeyError):
        return None, None
    for key, v in entries.items():
        c, b, name = key.split(":", 2)
        if int(c) == cfg and int(b) == batch and (name.startswith(kernel) or kernel.startswith(name)):
            _, sha = _source_of(kernel)
            date = v.get("date", table.get("_date"))
            if v.get("source_sha") and v.get("source_sha") == sha:
                return v, date
            return None, date
    return None, None


def roofline_of(per_kernel, cfg, batch):
    name = max(per_kernel, key=lambda k: per_kernel[k]["ms"])
    k = per_kernel[name]
    avg_ms = k["ms"] / k["launches"]
    gbs = (k["bytes"] / k["launches"]) / (avg_ms * 1e-3) / 1e9
    tflops = 2.0 * (k["macs"] / k["launches"]) / (avg_ms * 1e-3) / 1e12
    # the bound is the roof the kernel's algorithmic intensity puts it under
    alu = 2.0 * k["macs"] / max(k["bytes"], 1) > FP32_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    achieved, peak, unit = (tflops, FP32_PEAK_TFLOPS, "TFLOP/s") if alu else (gbs, HBM_PEAK_GBS, "GB/s")
    tr, tr_date = measured_traffic(cfg, batch, name)
    out = dict(bound="alu" if alu else "hbm", kernel=name, achieved=round(achieved, 3), peak=peak, unit=unit,
               frac=round(achieved / peak, 4), traffic=tr["fetch"] + tr["write"] if tr else None,
               traffic_fetch=tr["fetch"] if tr else None, traffic_write=tr["write"] if tr else None,
               traffic_profile_date=tr_date,
               launches_per_step=k["launches"],
               avg_launch_us=round(avg_ms * 1e3, 3), bytes_per_launch=k["bytes"] // k["launches"],
               flop_per_launch=2 * k["macs"] // k["launches"], algorithmic_gbs=round(gbs, 1),
               share_of_step=round(k["ms"] / sum(v["ms"] for v in per_kernel.values()), 3))
    if alu:
        out["peak_nonpacked"] = FP32_NONPACKED_TFLOPS
        out["frac_of_nonpacked"] = round(tflops / FP32_NONPACKED_TFLOPS, 4)
    return out


def step_roofline(prog, ms):
    """The whole step against what it must move and compute at the very least: only the program's inputs and results
    in HBM, every intermediate on chip."""
    if not getattr(prog, "min_bytes", 0):
        return None
    t_hbm = prog.min_bytes / (HBM_PEAK_GBS * 1e9)
    t_alu = prog.flops / (FP32_PEAK_TFLOPS * 1e12)
    t_bound = max(t_hbm, t_alu)
    return dict(min_bytes=prog.min_bytes, flops=prog.flops, bound="alu" if t_alu > t_hbm else "hbm",
                t_bound_us=round(t_bound * 1e6, 3), frac=round(t_bound / (ms * 1e-3), 4),
                min_bytes_gbs=round(prog.min_bytes / (ms * 1e-3) / 1e9, 1),
                tflops=round(prog.flops / (ms * 1e-3) / 1e12, 3),
                launch_bytes=prog.algorithmic_bytes())


def kernel_table(per_kernel):
    return {name: dict(launches=v["launches"], us_per_step=round(v["ms"] * 1e3, 2),
                       gbs=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else None)
            for name, v in per_kernel.items()}


# ---------------------------------------------------------------------------------------------- CPU oracle leg

def cpu_baseline(cfg, w, sample_ops, budget_s):
    """The CPU oracle as it stands on this host's cores, repeated on the same workload for about budget_s."""
    import oracle
    from oracle import programs as OP
    run = {1: OP.sum2_fwd, 2: OP.sum_chain_fwd_bwd, 3: OP.hashed_pipeline_fwd_bwd, 4: OP.dtkp_sum_chain,
           5: OP.grid_reach_fwd_bwd, 6: OP.product_chain_fwd_bwd, 7: OP.hwf_pipeline_dtkp, 8: OP.hwf_pipeline_damp}[cfg]
    want = int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1)

    def timed(threads, seconds):
        cores = oracle.set_threads(threads)
        run(w)                               # build + page in
        reps, t0 = 0, time.perf_counter()
        while True:
            run(w)
            reps += 1
            el = time.perf_counter() - t0
            if el >= seconds:
                return cores, reps, el

    cores, reps, el = timed(min(want, os.cpu_count() or 1), 0.75 * budget_s)
    _, reps1, el1 = timed(1, 0.25 * budget_s)
    oracle.set_threads(min(want, os.cpu_count() or 1))
    return dict(value=round(sample_ops * reps / el, 1), unit="sample-ops/s", cores=cores, kind="oracle",
                sample="%d full passes of the same workload (batch %d) in %.1f s" % (reps, w["batch"], el),
                single_thread_value=round(sample_ops * reps1 / el1, 1))


def near_ties(cfg, w):
    """Clamp decisions of the workload whose unclamped value, taken in float64 from the oracle's results, lies
    within 1e-6 of the clamp at 1: there the decision rests on the order of the float sum alone.
    Returns (count, decisions looked at), or None for a workload this is not defined for."""
    import numpy as np
    import oracle
    from oracle import programs as OP

    def count(pre64):
        return int((np.abs(np.asarray(pre64, np.float64) - 1.0) < NEAR_TIE).sum()), int(np.asarray(pre64).size)

    if cfg == 1:
        _, _, _, pre64 = oracle.damp_apply2_fwd(oracle.dense_to_triples(w["table"]), 10, 10, w["pa"], w["pb"], want_pre=True)
        return count(pre64)
    if cfg == 2:
        p, sym = w["p"], np.asarray(w["sym"], np.int32)
        acc, syms, n, tot = p[0], sym, 0, 0
        for t in range(1, p.shape[0]):
            tab = (syms[:, None] + sym[None, :]).astype(np.int32)
            syms, acc, _, pre64 = oracle.damp_apply2_fwd(oracle.dense_to_triples(tab), syms.size, sym.size, acc, p[t], want_pre=True)
            c = count(pre64)
            n, tot = n + c[0], tot + c[1]
        return n, tot
    if cfg == 3:
        tri = oracle.dense_to_triples(w["table"])
        s1, o1, _, pre64 = oracle.damp_apply2_fwd(tri, w["na"], w["nb"], w["pa"], w["pb"], want_pre=True)
        pred = w["keep"][s1]
        s2, _ = oracle.filter_plan(s1, pred)
        o2 = oracle.damp_filter_fwd(pred, o1)
        _, ia, ib = oracle.union_plan(s2, np.arange(w["n_out"], dtype=np.int32))
        both = (ia >= 0) & (ib >= 0)
        s = o2[:, ia[both]].astype(np.float64) + w["p2"][:, ib[both]].astype(np.float64)
        a, b = count(pre64), count(s)
        return a[0] + b[0], a[1] + b[1]
    if cfg == 4:
        res = OP.dtkp_sum_chain(w)
        n = tot = 0
        for _, _, pp, _ in res["stages"]:
            c = count(pp.astype(np.float64).sum(axis=-1))
            n, tot = n + c[0], tot + c[1]
        return n, tot
    if cfg == 5:
        res = OP.grid_reach_fwd_bwd(w)
        hist, p = res["hist"].astype(np.float64), w["p"].astype(np.float64)
        eu, ev = np.asarray(w["edge_u"]), np.asarray(w["edge_v"])
        n = tot = 0
        for t in range(w["rounds"]):
            r = hist[t]
            pre = r.copy()
            np.add.at(pre, (slice(None), ev), r[:, eu] * p)
            np.add.at(pre, (slice(None), eu), r[:, ev] * p)
            c = count(pre)
            n, tot = n + c[0], tot + c[1]
        return n, tot
    return None


# ---------------------------------------------------------------------------------------------- one workload

def build_program(GP, cfg, wl, chain):
    if chain in ("fused", "two-sweeps"):
        if cfg == 5:                         # the upstream gradient of these two workloads is an input: forward and
            return GP.GridReachFused(wl, one_launch=chain == "fused")            # backward share a launch
        if cfg == 3:
            return GP.HashedPipelineMerged(wl, one_launch=chain == "fused")
        fused = {2: GP.SumChainFused, 4: GP.DtkpSumChainFused}
        if cfg in fused:
            return fused[cfg](wl)
    return GP.make_program(cfg, wl)


def measure(cfg, args, torch, W, GP, batch=0):
    """One record: the workload as stated (or at `batch`), its B-scaled variant, the CPU oracle leg."""
    kw = dict(seed=args.seed)
    if batch:
        kw["batch"] = batch
    w = W.make_config(cfg, **kw)
    prog = build_program(GP, cfg, w, args.chain)
    mode = args.mode
    if mode == "auto":
        mode = "graph" if len(prog.launches) > 1 else "eager"
    run = make_runner(prog, torch, args.warmup, mode)
    ms, clock = time_step(run, torch, args.steps, args.regions, args.min_region_ms)
    per_kernel = time_launches(prog, torch, args.repeats)
    rec = {
        "config_id": cfg, "workload": w.name, "batch": prog.batch,
        "ms_per_step": round(ms, 6), "value": round(prog.sample_ops / (ms * 1e-3), 1), "unit": "sample-ops/s",
        "sample_ops_per_step": prog.sample_ops, "launches_per_step": len(prog.launches), "mode": mode,
        "chain": args.chain if cfg in (2, 3, 4, 5) else None, "clock": clock,
        "roofline": roofline_of(per_kernel, cfg, prog.batch),
        "step_roofline": step_roofline(prog, ms),
        "kernels": kernel_table(per_kernel),
    }
    if getattr(prog, "candidate_slots", 0):     # DTKP: proof pairs offered to the top-k lists, per second
        rec["candidate_slots_per_step"] = prog.candidate_slots
        rec["candidate_slots_per_s"] = round(prog.candidate_slots / (ms * 1e-3), 1)
    sample_ops = prog.sample_ops
    del prog, run
    torch.cuda.empty_cache()

    sb = SCALED_BATCH[cfg] if args.scaled_batch < 0 else args.scaled_batch
    if sb and not batch:
        kw["batch"] = sb
        ws = W.make_config(cfg, **kw)
        ps = build_program(GP, cfg, ws, args.chain)
        run_s = make_runner(ps, torch, 2, "eager")
        ms_s, clock_s = time_step(run_s, torch, max(args.scaled_steps, 20), 3, 0.0)
        pk = time_launches(ps, torch, 3, min_pair_ms=0.0)
        rs = roofline_of(pk, cfg, sb)
        rs.update(batch=sb, ms_per_step=round(ms_s, 5), value=round(ps.sample_ops / (ms_s * 1e-3), 1),
                  steps_per_region=clock_s["steps_per_region"], regions=clock_s["regions"],
                  step_roofline=step_roofline(ps, ms_s), kernels=kernel_table(pk))
        rec["scaled"] = rs
        del ps, ws, run_s
        torch.cuda.empty_cache()

    if args.cpu_seconds > 0:
        rec["cpu_baseline"] = cpu_baseline(cfg, w, sample_ops, args.cpu_seconds)
        nt = near_ties(cfg, w)
        if nt is not None:
            rec["near_ties"] = dict(count=nt[0], decisions=nt[1], within=NEAR_TIE)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=0, choices=[0, 1, 2, 3, 4, 5, 6, 7, 8],
                    help="measure this workload alone (1-5: the baseline configs; 6: Product-16 chain at B=256; 7 / 8: formula "
                         "pipeline of 7 positions at B=64 under DTKP-AM top-3 / DAMP); 0 = --configs")
    ap.add_argument("--configs", default="1,2,3,4,5", help="workloads of the default run, the headline being workload 2")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size (with --config)")
    ap.add_argument("--mode", default="auto", choices=["auto", "graph", "eager"],
                    help="how a step is issued: the launches one by one on the stream, or a HIP-graph replay of them; "
                         "auto = graph for steps of several launches, plain launches for a single-launch step (a graph "
                         "replay of one kernel only adds its own submission gap)")
    ap.add_argument("--chain", default="fused", choices=["fused", "two-sweeps", "per-op"],
                    help="configs 2-5: the fused entry points (dol_fold_apply2, dol_apply2_filter_union_forward_backward, "
                         "dol_dtkp_fold_apply2, dol_iterate_apply2_backward); two-sweeps: the same with configs 3 and 5 as a forward "
                         "and a backward launch (dol_apply2_filter_union + _backward, dol_iterate_apply2_ckpt + "
                         "dol_iterate_backward_ckpt); per-op: one dol_apply2 / dol_backward call per operator")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--regions", type=int, default=5, help="timed regions; the step time is their median")
    ap.add_argument("--min-region-ms", type=float, default=20.0, help="a region repeats its steps until it lasts this long")
    ap.add_argument("--repeats", type=int, default=20, help="fewest back-to-back launches per event pair in the roofline pass")
    ap.add_argument("--scaled-batch", type=int, default=-1, help="batch of the B-scaled variant (0 = skip)")
    ap.add_argument("--scaled-steps", type=int, default=20)
    ap.add_argument("--cpu-seconds", type=float, default=5.0, help="budget of the cpu_baseline leg per workload (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run the plain 1 GiB device copy (five times): the kernel of known size that the FETCH_SIZE / "
                         "WRITE_SIZE readings of a rocprofv3 --pmc run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no multi-GPU step (samples are independent, so a job shards by "
              "splitting the batch and replicating the symbol tables, with no exchange).  Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        print(json.dumps({"copy_mib": 1024, "reps": 5, "hbm_copy_gbs_measured": copy_rate(torch)}), flush=True)
        return

    import workloads as W
    from paper_2410_03348_amd import programs as GP

    if args.config:
        ids, head_id = [args.config], args.config
    else:
        ids = [int(x) for x in args.configs.split(",") if x]
        head_id = 2 if 2 in ids else ids[0]
    records = []
    for cfg in ids:
        print("[bench] workload %d ..." % cfg, file=sys.stderr, flush=True)
        records.append(measure(cfg, args, torch, W, GP, batch=args.batch if args.config else 0))
    head = next(r for r in records if r["config_id"] == head_id)

    out = {
        "metric": "batched apply sample-ops/sec (DAMP fwd+bwd, DTKP)",
        "value": head["value"],
        "unit": "sample-ops/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": head["workload"], "config_id": head_id, "batch": head["batch"],
                   "sample_ops_per_step": head["sample_ops_per_step"], "launches_per_step": head["launches_per_step"],
                   "mode": head["mode"], "seed": args.seed, "chain": head["chain"], "clock": head["clock"],
                   "algorithmic_bytes_per_step": head["step_roofline"]["launch_bytes"] if head["step_roofline"] else None},
        "roofline": dict(head["roofline"]),
        "kernels": head["kernels"],
    }
    out["roofline"]["hbm_copy_gbs_measured"] = copy_rate(torch)
    if "candidate_slots_per_s" in head:
        out["candidate_slots_per_s"] = head["candidate_slots_per_s"]
    if "scaled" in head:
        out["roofline_scaled"] = head["scaled"]
    if "cpu_baseline" in head:
        out["cpu_baseline"] = head["cpu_baseline"]
    if not args.config:
        out["configs"] = records
    else:
        for key in ("step_roofline", "near_ties"):
            if head.get(key) is not None:
                out[key] = head[key]
    out["date"] = datetime.date.today().isoformat()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
