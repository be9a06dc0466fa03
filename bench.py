#!/usr/bin/env python3
"""Benchmark of the Dolphin hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--batch B] [--mode auto|graph|eager]

A step is one pass of a whole program (all its operator launches, forward and backward) over one batch of
seeded synthetic input already resident in HBM.  The default program is workload 2, the Sum-15 DAMP
chain forward + backward at B=4096.  Prints ONE JSON line: whole-job sample-ops/s, the roofline of the
dominant kernel (measured live with HIP events on the launch stream), the same at a B-scaled variant of the
workload, and the CPU oracle timed on this host's cores.
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FP32_PEAK_TFLOPS = 157.3       # MI355X fp32 vector, published (256 CUs x 2.4 GHz x 128 lanes x 2 flop)
SCALED_BATCH = {1: 1 << 22, 2: 1 << 19, 3: 1 << 18, 4: 1 << 18, 5: 1 << 13, 6: 1 << 11, 7: 1 << 11, 8: 1 << 12}


def time_step(prog, torch, steps, warmup, mode):
    """Untimed warmup, then exactly `steps` steps between device synchronisations.  Returns ms per step."""
    for _ in range(max(warmup, 1)):
        prog.step()
    torch.cuda.synchronize()
    run = prog.step
    if mode == "graph":
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            prog.step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            prog.step()
        run = graph.replay
        for _ in range(max(warmup, 1)):
            run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def measured_copy_gbs(torch, mib=1024, reps=5):
    """Read + write rate of a plain device-to-device copy of `mib` MiB (the runtime's copy kernel), for setting the
    published HBM peak beside what a streaming kernel reaches on this device."""
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


def time_launches(prog, torch, repeats):
    """Average duration of every launch of a step: `repeats` back-to-back launches between two HIP events on
    the launch stream.  Returns {kernel: dict(launches, ms, bytes, macs)} summed over one step."""
    per_kernel = {}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for l in prog.launches:
        l.call()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(repeats):
            l.call()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / repeats
        k = per_kernel.setdefault(l.kernel, dict(launches=0, ms=0.0, bytes=0, macs=0))
        k["launches"] += 1
        k["ms"] += ms
        k["bytes"] += l.bytes
        k["macs"] += l.macs
    return per_kernel


def measured_traffic(cfg, batch, kernel):
    """HBM bytes per launch of `kernel` on this workload as the profiler's FETCH_SIZE / WRITE_SIZE counters gave
    them (a table written from separate rocprofv3 --pmc runs: the counters cannot be read from inside this
    program), or None when this workload was not profiled."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2410_03348_amd", "hbm_traffic.json")
    try:
        entries = json.load(open(path))["entries"]
    except (OSError, ValueError, KeyError):
        return None
    for key, v in entries.items():
        c, b, name = key.split(":", 2)
        if int(c) == cfg and int(b) == batch and (name.startswith(kernel) or kernel.startswith(name)):
            return v
    return None


def roofline_of(per_kernel, cfg, batch):
    name = max(per_kernel, key=lambda k: per_kernel[k]["ms"])
    k = per_kernel[name]
    avg_ms = k["ms"] / k["launches"]
    gbs = (k["bytes"] / k["launches"]) / (avg_ms * 1e-3) / 1e9
    tflops = 2.0 * (k["macs"] / k["launches"]) / (avg_ms * 1e-3) / 1e12
    # the bound is the roof the kernel's algorithmic intensity puts it under
    alu = 2.0 * k["macs"] / max(k["bytes"], 1) > FP32_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    achieved, peak, unit = (tflops, FP32_PEAK_TFLOPS, "TFLOP/s") if alu else (gbs, HBM_PEAK_GBS, "GB/s")
    tr = measured_traffic(cfg, batch, name)
    return dict(bound="alu" if alu else "hbm", kernel=name, achieved=round(achieved, 3), peak=peak, unit=unit,
                frac=round(achieved / peak, 4), traffic=tr["fetch"] + tr["write"] if tr else None,
                traffic_fetch=tr["fetch"] if tr else None, traffic_write=tr["write"] if tr else None,
                launches_per_step=k["launches"],
                avg_launch_us=round(avg_ms * 1e3, 3), bytes_per_launch=k["bytes"] // k["launches"],
                flop_per_launch=2 * k["macs"] // k["launches"], algorithmic_gbs=round(gbs, 1),
                share_of_step=round(k["ms"] / sum(v["ms"] for v in per_kernel.values()), 3))


def kernel_table(per_kernel):
    return {name: dict(launches=v["launches"], us_per_step=round(v["ms"] * 1e3, 2),
                       gbs=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else None)
            for name, v in per_kernel.items()}


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
    return dict(value=round(sample_ops * reps / el, 1), unit="sample-ops/s", cores=cores, kind="oracle",
                sample="%d full passes of the same workload (batch %d) in %.1f s" % (reps, w["batch"], el),
                single_thread_value=round(sample_ops * reps1 / el1, 1))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5, 6, 7, 8],
                    help="1-5: the baseline configs; 6: Product-16 chain at B=256; 7 / 8: formula pipeline of 7 positions "
                         "at B=64 under DTKP-AM top-3 / DAMP (6-8: per-operator calls)")
    ap.add_argument("--batch", type=int, default=0, help="override the config's batch size")
    ap.add_argument("--mode", default="auto", choices=["auto", "graph", "eager"],
                    help="how a step is issued: the launches one by one on the stream, or a HIP-graph replay of them; "
                         "auto = graph for steps of several launches, plain launches for a single-launch step (a graph "
                         "replay of one kernel only adds its own submission gap)")
    ap.add_argument("--chain", default="fused", choices=["fused", "per-op"],
                    help="configs 2-5: the fused entry points (dol_fold_apply2, dol_filter_union, dol_dtkp_fold_apply2, dol_iterate_*), or one dol_apply2 / "
                         "dol_backward call per operator")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--repeats", type=int, default=20, help="back-to-back launches per event pair in the roofline pass")
    ap.add_argument("--scaled-batch", type=int, default=-1, help="batch of the B-scaled variant (0 = skip)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="budget of the cpu_baseline leg (0 = skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the path has no multi-GPU step (samples are independent, so a job shards by "
              "splitting the batch and replicating the symbol tables, with no exchange).  Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W
    from paper_2410_03348_amd import programs as GP

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = args.config
    kw = dict(seed=args.seed)
    if args.batch:
        kw["batch"] = args.batch
    w = W.make_config(cfg, **kw)

    def build(wl):
        if args.chain == "fused" and cfg == 2:
            return GP.SumChainFused(wl)
        if args.chain == "fused" and cfg == 5:
            return GP.GridReachFused(wl)
        if args.chain == "fused" and cfg == 3:
            return GP.HashedPipelineFused(wl)
        if args.chain == "fused" and cfg == 4:
            return GP.DtkpSumChainFused(wl)
        return GP.make_program(cfg, wl)
    prog = build(w)
    if args.mode == "auto":
        args.mode = "graph" if len(prog.launches) > 1 else "eager"
    ms = time_step(prog, torch, args.steps, args.warmup, args.mode)
    per_kernel = time_launches(prog, torch, args.repeats)
    roof = roofline_of(per_kernel, cfg, prog.batch)

    out = {
        "metric": "batched apply sample-ops/sec (DAMP fwd+bwd, DTKP)",
        "value": round(prog.sample_ops / (ms * 1e-3), 1),
        "unit": "sample-ops/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "config_id": cfg, "batch": prog.batch, "sample_ops_per_step": prog.sample_ops,
                   "launches_per_step": len(prog.launches), "mode": args.mode, "seed": args.seed,
                   "chain": args.chain if cfg in (2, 3, 4, 5) else None,
                   "algorithmic_bytes_per_step": prog.algorithmic_bytes()},
        "roofline": roof,
        "kernels": kernel_table(per_kernel),
    }
    out["roofline"]["hbm_copy_gbs_measured"] = measured_copy_gbs(torch)
    if getattr(prog, "candidate_slots", 0):     # DTKP: proof pairs offered to the top-k lists, per second
        out["config"]["candidate_slots_per_step"] = prog.candidate_slots
        out["candidate_slots_per_s"] = round(prog.candidate_slots / (ms * 1e-3), 1)

    sb = SCALED_BATCH[cfg] if args.scaled_batch < 0 else args.scaled_batch
    if sb:
        del prog
        torch.cuda.empty_cache()
        kw["batch"] = sb
        ws = W.make_config(cfg, **kw)
        ps = build(ws)
        ms_s = time_step(ps, torch, 3, 1, "eager")
        pk = time_launches(ps, torch, 3)
        rs = roofline_of(pk, cfg, sb)
        rs.update(batch=sb, ms_per_step=round(ms_s, 4), value=round(ps.sample_ops / (ms_s * 1e-3), 1),
                  step_gbs=round(ps.algorithmic_bytes() / (ms_s * 1e-3) / 1e9, 1), kernels=kernel_table(pk))
        out["roofline_scaled"] = rs
        del ps, ws
        torch.cuda.empty_cache()

    if args.cpu_seconds > 0:
        out["cpu_baseline"] = cpu_baseline(cfg, w, out["config"]["sample_ops_per_step"], args.cpu_seconds)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
