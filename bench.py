#!/usr/bin/env python3
"""Benchmark of the two-stage depth-compression DP on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--shape 0]

One step = one pass of the whole hot path over one batch of synthetic input
that is already resident in HBM: dpc_stage1_minplus, dpc_stage2_knapsack,
dpc_backtrack, queued on one stream.  The default workload is the stress
configuration (B=64, L=200, P=16000, dense feasibility, M and K stored, set
recovery at every budget that is a multiple of 100), the one the throughput
target is quoted on.  Prints ONE JSON line.

  value        nominal relax-ops per second, B*L^2*P / step time, as the metric
               is named; `exact_relax_ops_per_s` counts the candidates that
               exist, B*P*L(L+1)/2, and is what the roofline uses.
  roofline     stage-2 kernel(s): plain-VALU bound.  One relax = 1 add,
               1 compare, 2 selects = 4 lane-ops (2 when K is not stored);
               peak = 256 CU x 64 lanes/clk x 2.4 GHz = 39.3 T lane-ops/s
               (the 157.3 TFLOP/s fp32 vector figure without the FMA and
               packed factors of 2).  Duration from HIP events on the launch
               stream around dpc_stage2_knapsack in every timed step (the only
               events in the timed region; stage 1 and set recovery are timed
               in further steps after it).
               `frac` counts 4 lane-ops per candidate (the update taken
               one candidate at a time) whatever the kernel issues, so it
               can pass 1; `variant_floor_ops` / `frac_of_variant_floor`
               count what the arithmetic of the main loop of the kernel
               shape that ran needs at least, `issued_valu_per_relax` /
               `frac_issued` what the counters saw.
  cpu_baseline the CPU oracle, as it stands, on every instance and query of the
               same workload, one instance per host thread (`cores` threads
               of `host_cores`).
  parity       the GPU buffers as the last step left them (every step solves the
               same inputs) against that oracle run, element by element,
               tolerance 0; a mismatch makes the exit status 1.
  per_config   (default run only) workloads 1-4 timed and checked the same way.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "DP relax-ops/sec (B·L²·P) + batch solve latency ms, 1×MI355X"
VALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9        # 39.3e12
# Figures that come from the committed rocprofv3 summaries, not from this run
# (counters cannot be read from inside the process): HBM bytes per stage-2
# launch (FETCH_SIZE / WRITE_SIZE runs) and VALU instructions issued per
# candidate (SQ_INSTS_VALU x 64 lanes / exact candidates), keyed by config.
PROFILED = {
    3: {"file": "profiles/stage2_cfg3.md", "traffic_bytes": 0.929e9,
        "issued_valu_per_relax": 4.41},
    4: {"file": "profiles/stage2_cfg4.md", "traffic_bytes": 1.806e9,
        "issued_valu_per_relax": 3.84},
    5: {"file": "profiles/stage2_wave_kernel_cfg5.md", "traffic_bytes": 6.643e9,
        "issued_valu_per_relax": 3.39},
}


def variant_floor_ops(L, P, store_K):
    """VALU instructions per candidate that the arithmetic of the main loop of the
    kernel shape the library picks for (L, P) cannot go below.  With
    back-pointers, tables wider than 512 budgets take two predecessor rows per
    step: 2 adds, 1 three-way max, 1 compare, 1 byte select per two candidates =
    2.5; narrower ones take one: add, compare, 2 selects = 4.  Without
    back-pointers: 2 adds + 1 three-way max = 1.5 for 16-row groups, add + max = 2
    for 8-row groups."""
    if store_K:
        return 2.5 if P > 512 else 4.0
    return 1.5 if (L >= 64 and P > 512) else 2.0


class Workload:
    """One named workload resident on the GPU, with its buffers."""

    def __init__(self, cid, seed, store_K, torch, api, inputs):
        self.cfg = cfg = inputs.CONFIGS[cid]
        dev = torch.device("cuda:0")
        self.T, self.I, base = inputs.make_batch(cfg, seed=seed)
        self.qi, self.qt = inputs.budgets(cfg, base)
        self.Td, self.Id = torch.from_numpy(self.T).to(dev), torch.from_numpy(self.I).to(dev)
        self.qid, self.qtd = torch.from_numpy(self.qi).to(dev), torch.from_numpy(self.qt).to(dev)
        self.buf = api.Buffers(cfg.B, cfg.L, cfg.P, len(self.qi), store_K=store_K)


def time_workload(w, args, torch, api, np, steps, warmup, fused=False, graph=False):
    """W untimed and K timed steps of the whole path; -> (ms per step by the host
    clock around the K steps, per-stage ms from events on the launch stream).
    The timed steps carry one event pair each, around stage 2 (the roofline's
    duration); the durations of stage 1 and of the set recovery come from K more
    steps after the timed region, which carry an event at every stage boundary."""
    buf, stream = w.buf, torch.cuda.current_stream()
    one_launch = fused and 0 < len(w.qi) <= api.ONE_LAUNCH_QUERIES_PER_INSTANCE * w.cfg.B

    def step(ev=None, which=()):
        def mark(x):
            if ev is not None and x in which:
                ev[x].record(stream)
        mark(0)
        if fused and one_launch:
            # the whole path in one kernel: its time is reported as stage 2
            mark(1)
            api.dpc_solve_fused(w.Td, w.Id, buf.Topt, buf.split, buf.M, buf.K, w.qid, w.qtd, buf.A,
                                buf.A_len, buf.S, buf.S_len, buf.obj, buf.lat, buf.status)
            mark(2)
            mark(3)
            return
        if fused:
            mark(1)                          # (stage 1 runs inside the one kernel)
            api.dpc_stage12_fused(w.Td, w.Id, buf.Topt, buf.split, buf.M, buf.K)
        else:
            api.dpc_stage1_minplus(w.Td, buf.Topt, buf.split)
            mark(1)
            api.dpc_stage2_knapsack(buf.Topt, w.Id, buf.M, buf.K, buf.workspace, shape=args.shape)
        mark(2)
        api.dpc_backtrack(buf.Topt, buf.split, w.Id, buf.M, buf.K, w.qid, w.qtd, buf.A, buf.A_len,
                          buf.S, buf.S_len, buf.obj, buf.lat, buf.status)
        mark(3)

    S2_ONLY, ALL = (1, 2), (0, 1, 2, 3)
    for _ in range(warmup):
        step()
    api.dpc_stage2_check(buf.workspace)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    torch.cuda.synchronize()
    if graph:
        # (the stage-2 events are recorded inside the graph once; the replays are timed as a whole)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        g.replay()
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        t0 = time.perf_counter()
        for k in range(steps):
            evs[k][0].record(stream)
            g.replay()
            for x in (1, 2, 3):
                evs[k][x].record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        api.dpc_stage2_check(buf.workspace)
        seg = [[e[x].elapsed_time(e[x + 1]) for e in evs] for x in range(3)]
        return (t1 - t0) * 1e3 / steps, {
            "stage1": float(np.mean(seg[0])), "stage2": float(np.mean(seg[1])),
            "stage2_min": float(np.min(seg[1])), "backtrack": float(np.mean(seg[2]))}
    t0 = time.perf_counter()
    for k in range(steps):
        step(evs[k], S2_ONLY)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    api.dpc_stage2_check(buf.workspace)
    ms_step = (t1 - t0) * 1e3 / steps
    s2 = [e[1].elapsed_time(e[2]) for e in evs]
    stage_ms = {"stage2": float(np.mean(s2)), "stage2_min": float(np.min(s2))}
    # the other stages: the same K steps again, after the timed region, with an
    # event at every stage boundary
    evs2 = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    for k in range(steps):
        step(evs2[k], ALL)
    torch.cuda.synchronize()
    stage_ms["stage1"] = float(np.mean([e[0].elapsed_time(e[1]) for e in evs2]))
    stage_ms["backtrack"] = float(np.mean([e[2].elapsed_time(e[3]) for e in evs2]))
    # and once more with no events in the stream at all: on the small workloads
    # an event record takes as long as a kernel
    t0 = time.perf_counter()
    for k in range(steps):
        step()
    torch.cuda.synchronize()
    stage_ms["step_without_events"] = (time.perf_counter() - t0) * 1e3 / steps
    return ms_step, stage_ms


def oracle_leg(w, np, oracle, cores, want_K):
    """The oracle, as it stands, on every instance and query of the workload (one
    instance per host thread), timed; then the GPU buffers of the last step
    against it, element by element, tolerance 0.  -> (seconds, parity dict)."""
    cfg, buf = w.cfg, w.buf
    tc0 = time.perf_counter()
    To, sp, Mo, Ko = oracle.solve_batch(w.T, w.I, cfg.P, want_K=True, threads=cores)
    res = [oracle.backtrack(To[b], sp[b], w.I[b], Mo[b], Ko[b] if want_K else None, int(t))
           for b, t in zip(w.qi, w.qt)]
    tc1 = time.perf_counter()
    bad = 0
    bad += int((buf.Topt.cpu().numpy() != To).sum()) + int((buf.split.cpu().numpy() != sp).sum())
    for b in range(cfg.B):                       # instance by instance: the tables are large
        bad += int((buf.M[b].cpu().numpy().view(np.uint32) != Mo[b].view(np.uint32)).sum())
        if buf.K is not None:
            bad += int((buf.K[b].cpu().numpy() != Ko[b]).sum())
    g = {k: getattr(buf, k).cpu().numpy() for k in ("A", "S", "A_len", "S_len", "obj", "lat", "status")}
    qbad = 0
    for q, r in enumerate(res):
        same = (g["status"][q] == r["status"] and g["A_len"][q] == r["A_len"]
                and g["S_len"][q] == r["S_len"] and g["lat"][q] == r["lat"]
                and g["obj"][q:q + 1].view(np.uint32)[0] == np.array([r["obj"]], np.float32).view(np.uint32)[0])
        if same and r["status"] == 0:
            same = (list(g["A"][q][:r["A_len"]]) == list(r["A"])
                    and list(g["S"][q][:r["S_len"]]) == list(r["S"]))
        qbad += 0 if same else 1
    cells = cfg.B * (cfg.L + 1) * cfg.P
    parity = {"instances": cfg.B, "queries": len(res), "table_cells": cells,
              "compared": "Topt, split, M" + (", K" if buf.K is not None else "") +
                          "; status, A, S, objective, latency of every query",
              "mismatches": bad + qbad}
    return tc1 - tc0, parity


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--shape", type=int, default=0,
                    help="stage-2 kernel shape through the test hook (0 = the library's choice)")
    ap.add_argument("--no-K", action="store_true", help="do not store back-pointers")
    ap.add_argument("--no-cpu", action="store_true",
                    help="skip the cpu_baseline leg and the parity check against it")
    ap.add_argument("--no-per-config", action="store_true",
                    help="skip the timings of workloads 1-4 that follow the headline one")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--ext", action="store_true",
                    help="time the extended solver (Appendix B: Algorithms 1, 3, 4 and set "
                         "recovery) on the flag-dependent version of --config (default 3, the "
                         "MobileNetV2-shaped batch) instead of the headline workload")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph once and time its replays")
    ap.add_argument("--fused", action="store_true",
                    help="the single-launch path for small instances (L <= 63, P <= 2048): "
                         "dpc_solve_fused when there are few queries per instance, else "
                         "dpc_stage12_fused + dpc_backtrack")
    ap.add_argument("--sweep", action="store_true",
                    help="time a sweep over the normalisation constant alpha: shift, solve, "
                         "trade-off curves, set recovery, latency merged at A (cfg3 shape by default)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device copy (reference point for the "
                         "FETCH_SIZE / WRITE_SIZE counters), print its size and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the instances shard trivially over "
              "GPUs with no exchange, see DESIGN.md); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2301_12187_amd import api, inputs

    if args.copy_calibration:
        n = 1 << 28                                   # 2^28 floats = 1 GiB read + 1 GiB written
        src = torch.ones(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 4 * n, "copy_calibration_bytes_written": 4 * n,
                          "launches": 3}))
        return

    if args.ext:
        return bench_ext(args, np, torch, api, inputs)
    if args.sweep:
        return bench_sweep(args, np, torch, api, inputs)
    torch.cuda.set_device(torch.device("cuda:0"))
    store_K = not args.no_K
    host_cores = os.cpu_count() or 1
    cores = min(16, host_cores)                  # the GPU machine gives one job 16 cores' worth
    w = Workload(args.config, args.seed, store_K, torch, api, inputs)
    cfg = w.cfg

    if args.fused and not api.dpc_stage12_fused_supported(cfg.L, cfg.P):
        print(f"bench.py --fused: L = {cfg.L}, P = {cfg.P} is outside the single-launch path",
              file=sys.stderr)
        sys.exit(2)

    ms_step, stage_ms = time_workload(w, args, torch, api, np, args.steps, args.warmup,
                                      fused=args.fused, graph=args.graph)
    exact = inputs.relax_ops_exact(cfg.B, cfg.L, cfg.P)
    nominal = inputs.relax_ops_nominal(cfg.B, cfg.L, cfg.P)
    s2_avg = stage_ms["stage2"]
    ops_per_relax = 4 if store_K else 2
    achieved = ops_per_relax * exact / (s2_avg * 1e-3)
    floor_ops = variant_floor_ops(cfg.L, cfg.P, store_K)
    prof = PROFILED.get(args.config) if (store_K and args.shape == 0 and not args.fused) else None

    out = {
        "metric": METRIC,
        "value": nominal / (ms_step * 1e-3),
        "unit": "relax-ops/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "L": cfg.L, "P": cfg.P,
                   "queries": int(len(w.qi)), "store_K": store_K,
                   "stage2_shape": args.shape, "fused_stage12": bool(args.fused),
                   "graph_replay": bool(args.graph),
                   "seed": args.seed},
        "exact_relax_ops_per_s": exact / (ms_step * 1e-3),
        "stage2_exact_relax_ops_per_s": exact / (s2_avg * 1e-3),
        "stage_ms": stage_ms,
        "feasible_queries": int((w.buf.status == 0).sum().item()),
        "host_cores": host_cores,
        "roofline": {
            "bound": "alu", "kernel": "stage 2 (dpc_stage2_knapsack)",
            "achieved": achieved / 1e12, "peak": VALU_PEAK_LANE_OPS / 1e12,
            "unit": "TOP/s", "frac": achieved / VALU_PEAK_LANE_OPS,
            # `frac` counts the update one candidate at a time (add, compare, two
            # selects); the kernel shape that ran issues fewer in its main loop:
            "ops_per_relax": ops_per_relax,
            "variant_floor_ops": floor_ops,
            "frac_of_variant_floor": floor_ops * exact / (s2_avg * 1e-3) / VALU_PEAK_LANE_OPS,
            "issued_valu_per_relax": prof["issued_valu_per_relax"] if prof else None,
            # the VALU instructions the kernel issued, as a fraction of the peak
            "frac_issued": (prof["issued_valu_per_relax"] * exact / (s2_avg * 1e-3) / VALU_PEAK_LANE_OPS)
                           if prof else None,
            "traffic": prof["traffic_bytes"] if prof else None,
            "traffic_source": (prof["file"] + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, not this run)")
                              if prof else None,
        },
    }

    ok = True
    if not args.no_cpu:
        import oracle
        secs, parity = oracle_leg(w, np, oracle, cores, store_K)
        out["cpu_baseline"] = {
            "value": nominal / secs, "unit": "relax-ops/s", "cores": min(cores, cfg.B),
            "host_cores": host_cores, "kind": "oracle",
            "sample": f"all {cfg.B} instances and {len(w.qi)} queries of {cfg.name}, all stages, "
                      f"{secs:.2f} s wall",
        }
        out["parity"] = parity
        ok = ok and parity["mismatches"] == 0

    if not args.no_per_config and args.config == 5 and not (args.fused or args.graph):
        # the other four workloads, timed the same way (and checked the same way)
        del w
        torch.cuda.empty_cache()
        per = {}
        for cid in (1, 2, 3, 4):
            wc = Workload(cid, args.seed, store_K, torch, api, inputs)
            c = wc.cfg
            ms_c, st_c = time_workload(wc, args, torch, api, np, args.steps, args.warmup)
            ex = inputs.relax_ops_exact(c.B, c.L, c.P)
            fl = variant_floor_ops(c.L, c.P, store_K)
            rate = ex / (st_c["stage2"] * 1e-3)
            per[str(cid)] = {
                "workload": c.name, "ms_step": ms_c, "stage_ms": st_c,
                "nominal_relax_per_s": inputs.relax_ops_nominal(c.B, c.L, c.P) / (ms_c * 1e-3),
                "stage2_exact_relax_per_s": rate,
                "frac": ops_per_relax * rate / VALU_PEAK_LANE_OPS,
                "variant_floor_ops": fl, "frac_of_variant_floor": fl * rate / VALU_PEAK_LANE_OPS,
            }
            if store_K and args.shape == 0 and cid in PROFILED:
                per[str(cid)]["issued_valu_per_relax"] = PROFILED[cid]["issued_valu_per_relax"]
                per[str(cid)]["traffic"] = PROFILED[cid]["traffic_bytes"]
                per[str(cid)]["traffic_source"] = PROFILED[cid]["file"] + " (rocprofv3 --pmc, not this run)"
            if not args.no_cpu:
                import oracle
                secs, parity = oracle_leg(wc, np, oracle, cores, store_K)
                per[str(cid)]["cpu_oracle_s"] = secs
                per[str(cid)]["parity"] = parity
                ok = ok and parity["mismatches"] == 0
            if cid in (1, 2) and api.dpc_stage12_fused_supported(c.L, c.P):
                # the single-launch path for small instances, timed and checked the same way
                ms_f, st_f = time_workload(wc, args, torch, api, np, args.steps, args.warmup, fused=True)
                per[str(cid)]["single_launch_path"] = {"ms_step": ms_f, "stage_ms": st_f}
                if not args.no_cpu:
                    _, parity_f = oracle_leg(wc, np, oracle, cores, store_K)
                    per[str(cid)]["single_launch_path"]["parity"] = parity_f
                    ok = ok and parity_f["mismatches"] == 0
            del wc
            torch.cuda.empty_cache()
        out["per_config"] = per
    print(json.dumps(out))
    if not ok:
        print("bench.py: the GPU results differ from the oracle's", file=sys.stderr)
        sys.exit(1)


def bench_ext(args, np, torch, api, inputs):
    """Extended solver: one step = dpc_stage1_minplus + dpc_ext_importance_maxplus +
    dpc_ext_knapsack + dpc_ext_backtrack.  A relax-op is one candidate
    (instance, k', alpha', l, a, t) of Algorithm 4: four per pair (k', l) and budget."""
    cid = 3 if args.config == 5 else args.config
    cfg = inputs.CONFIGS[cid]
    if cfg.L > api.DPC_EXT_MAX_L:
        print(f"bench.py --ext: L = {cfg.L} exceeds the extended solver's limit", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    T, I4, base = inputs.make_ext_batch(cfg, seed=args.seed)
    qi, qt = inputs.budgets(cfg, base)
    Td, Id = torch.from_numpy(T).to(dev), torch.from_numpy(I4).to(dev)
    qid, qtd = torch.from_numpy(qi).to(dev), torch.from_numpy(qt).to(dev)
    buf = api.ExtBuffers(cfg.B, cfg.L, cfg.P, len(qi))
    stream = torch.cuda.current_stream()
    for _ in range(args.warmup):
        api.ext_solve(Td, Id, qid, qtd, buf)
    api.dpc_ext_check(cfg.B, cfg.L, cfg.P, buf.workspace)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for ev in evs:
        ev[0].record(stream)
        api.dpc_stage1_minplus(Td, buf.Topt, buf.split)
        ev[1].record(stream)
        api.dpc_ext_importance_maxplus(Id, buf.Iopt, buf.bsplit)
        ev[2].record(stream)
        api.dpc_ext_knapsack(buf.Topt, buf.Iopt, buf.D, buf.Kx, buf.workspace)
        ev[3].record(stream)
        api.dpc_ext_backtrack(buf.Topt, buf.split, buf.bsplit, buf.D, buf.Kx, qid, qtd, buf.A,
                              buf.A_len, buf.S, buf.S_len, buf.Bs, buf.B_len, buf.obj, buf.lat,
                              buf.a_last, buf.status)
        ev[4].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    api.dpc_ext_check(cfg.B, cfg.L, cfg.P, buf.workspace)
    ms_step = (t1 - t0) * 1e3 / args.steps
    seg = [[e[x].elapsed_time(e[x + 1]) for e in evs] for x in range(4)]
    exact = 4 * inputs.relax_ops_exact(cfg.B, cfg.L, cfg.P)
    s2 = float(np.mean(seg[2]))
    out = {
        "metric": "extended-solver relax-ops/sec (4 per pair and budget) + batch solve latency ms, 1xMI355X",
        "value": exact / (ms_step * 1e-3), "unit": "relax-ops/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "extended solver on " + cfg.name, "B": cfg.B, "L": cfg.L, "P": cfg.P,
                   "queries": int(len(qi)), "seed": args.seed},
        "stage_ms": {"stage1": float(np.mean(seg[0])), "importance_maxplus": float(np.mean(seg[1])),
                     "knapsack": s2, "backtrack": float(np.mean(seg[3]))},
        "feasible_queries": int((buf.status == 0).sum().item()),
        "roofline": {"bound": "alu", "kernel": "Algorithm 4 (dpc_ext_knapsack)",
                     "achieved": 4 * exact / (s2 * 1e-3) / 1e12, "peak": VALU_PEAK_LANE_OPS / 1e12,
                     "unit": "TOP/s", "frac": 4 * exact / (s2 * 1e-3) / VALU_PEAK_LANE_OPS,
                     "ops_per_relax": 4, "traffic": None},
    }
    if not args.no_cpu:
        import oracle
        cores = min(16, os.cpu_count() or 1)
        nb = cfg.B
        tc0 = time.perf_counter()
        res = oracle.ext_solve_batch(T[:nb], I4[:nb], cfg.P, threads=cores)
        for b, t in zip(qi[qi < nb], qt[qi < nb]):
            oracle.ext_backtrack(res[0][b], res[1][b], res[3][b], res[4][b], res[5][b], int(t))
        tc1 = time.perf_counter()
        out["cpu_baseline"] = {"value": 4 * inputs.relax_ops_exact(nb, cfg.L, cfg.P) / (tc1 - tc0),
                               "unit": "relax-ops/s", "cores": min(cores, nb), "kind": "oracle",
                               "sample": f"{nb} of {cfg.B} instances, all stages, {tc1 - tc0:.2f} s wall"}
    print(json.dumps(out))


def bench_sweep(args, np, torch, api, inputs):
    """Sweep over the normalisation constant: one step = dpc_importance_shift (n_raw tables x
    n_alpha constants -> B instances) + stage 1 (once per raw table: the copies share it) +
    stage 2 + dpc_front + dpc_front_queries + dpc_backtrack at every point of every trade-off
    curve + dpc_chain_latency at A."""
    cid = 3 if args.config == 5 else args.config
    cfg = inputs.CONFIGS[cid]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n_alpha = 16 if cfg.B >= 16 else 1
    T0, I_raw, base, alphas = inputs.make_sweep_batch(cfg, seed=args.seed, n_alpha=n_alpha)
    n_raw = T0.shape[0]
    B = n_raw * n_alpha
    T = np.repeat(T0, n_alpha, axis=0)
    Td = torch.from_numpy(T).to(dev)            # (per instance: dpc_chain_latency indexes it by query)
    T0d = torch.from_numpy(T0).to(dev)
    Topt = torch.empty((n_raw, cfg.L + 1, cfg.L + 1), dtype=torch.int32, device=dev)
    split = torch.empty((n_raw, cfg.L + 1, cfg.L + 1), dtype=torch.uint8, device=dev)
    Ird = torch.from_numpy(I_raw).to(dev)
    ald = torch.from_numpy(alphas).to(dev)
    # one query per point of every curve; the list is built on the device, so its
    # room is fixed (64 points per instance on average) and the unused tail holds
    # instance -1, which set recovery answers with "bad query" at once
    qcap = 64 * B
    qid = torch.full((qcap,), -1, dtype=torch.int32, device=dev)
    qtd = torch.zeros((qcap,), dtype=torch.int32, device=dev)
    qn = torch.zeros((1,), dtype=torch.int32, device=dev)
    buf = api.Buffers(B, cfg.L, cfg.P, qcap, store_K=True)
    Id = torch.empty((B, cfg.L + 1, cfg.L + 1), dtype=torch.float32, device=dev)
    cap = 256
    ft = torch.empty((B, cap), dtype=torch.int32, device=dev)
    fo = torch.empty((B, cap), dtype=torch.float32, device=dev)
    fl = torch.empty((B,), dtype=torch.int32, device=dev)
    latA = torch.empty((qcap,), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    names = ["importance_shift", "stage1", "stage2", "front", "front_queries", "backtrack",
             "chain_latency"]

    def step(ev=None):
        calls = [
            lambda: api.dpc_importance_shift(Ird, ald, Id),
            lambda: api.dpc_stage1_minplus(T0d, Topt, split),
            lambda: api.dpc_stage2_knapsack_shared(n_alpha, Topt, Id, buf.M, buf.K, buf.workspace),
            lambda: api.dpc_front(buf.M, ft, fo, fl),
            lambda: api.dpc_front_queries(ft, fl, qid, qtd, qn),
            lambda: api.dpc_backtrack_shared(n_alpha, Topt, split, Id, buf.M, buf.K, qid, qtd, buf.A,
                                             buf.A_len, buf.S, buf.S_len, buf.obj, buf.lat, buf.status),
            lambda: api.dpc_chain_latency(Td, qid, buf.A, buf.A_len, latA),
        ]
        for x, call in enumerate(calls):
            if ev:
                ev[x].record(stream)
            call()
        if ev:
            ev[len(calls)].record(stream)

    for _ in range(args.warmup):
        step()
    api.dpc_stage2_check(buf.workspace)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(8)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for ev in evs:
        step(ev)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    api.dpc_stage2_check(buf.workspace)
    ms_step = (t1 - t0) * 1e3 / args.steps
    seg = {n: float(np.mean([e[x].elapsed_time(e[x + 1]) for e in evs])) for x, n in enumerate(names)}
    exact = inputs.relax_ops_exact(B, cfg.L, cfg.P)
    ok = buf.status == 0
    out = {
        "metric": "sweep over the normalisation constant: relax-ops/sec (B*L^2*P) + batch latency ms, 1xMI355X",
        "value": inputs.relax_ops_nominal(B, cfg.L, cfg.P) / (ms_step * 1e-3), "unit": "relax-ops/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"alpha sweep on {cfg.name}", "raw_tables": n_raw, "alphas": n_alpha,
                   "B": B, "L": cfg.L, "P": cfg.P, "queries": int(qn.item()), "query_room": qcap,
                   "front_cap": cap,
                   "seed": args.seed},
        "stage_ms": seg,
        "feasible_queries": int(ok.sum().item()),
        "mean_front_points": float(fl.float().mean().item()),
        # merging at A alone needs every block between two kept activations to be one layer
        "mergeable_at_A": int((ok & (latA < api.DPC_INF)).sum().item()),
        "mean_latency_merged_at_A_over_S": float(
            (latA[ok & (latA < api.DPC_INF)].double()
             / buf.lat[ok & (latA < api.DPC_INF)].double().clamp(min=1)).mean().item()),
        "roofline": {"bound": "alu", "kernel": "stage 2 (dpc_stage2_knapsack)",
                     "achieved": 4 * exact / (seg["stage2"] * 1e-3) / 1e12,
                     "peak": VALU_PEAK_LANE_OPS / 1e12, "unit": "TOP/s",
                     "frac": 4 * exact / (seg["stage2"] * 1e-3) / VALU_PEAK_LANE_OPS,
                     "ops_per_relax": 4, "traffic": None},
    }
    if not args.no_cpu:
        import oracle
        cores = min(16, os.cpu_count() or 1)
        tc0 = time.perf_counter()
        Is = np.stack([oracle.importance_shift(I_raw[b // n_alpha], alphas[b % n_alpha])[0]
                       for b in range(B)])
        To, sp, Mo, Ko = oracle.solve_batch(T, Is, cfg.P, want_K=True, threads=cores)
        fts = np.full((B, cap), -1, np.int32)
        fls = np.zeros(B, np.int32)
        for b in range(B):
            t_, _, n_ = oracle.front(Mo[b, cfg.L], cap)
            fts[b, :len(t_)] = t_
            fls[b] = n_
        qi, qt, _ = oracle.front_queries(fts, fls, qcap)
        for b, t in zip(qi, qt):
            r = oracle.backtrack(To[b], sp[b], Is[b], Mo[b], Ko[b], int(t))
            oracle.chain_latency(T[b], None if r["status"] else r["A"])
        tc1 = time.perf_counter()
        out["cpu_baseline"] = {"value": inputs.relax_ops_nominal(B, cfg.L, cfg.P) / (tc1 - tc0),
                               "unit": "relax-ops/s", "cores": min(cores, B), "kind": "oracle",
                               "sample": f"all {B} instances, all steps, {tc1 - tc0:.2f} s wall"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
