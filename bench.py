#!/usr/bin/env python3
"""Benchmark of the two-stage depth-compression DP on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--variant 0]

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
               stream around dpc_stage2_knapsack in every timed step.
  cpu_baseline the CPU oracle, as it stands, on a bounded sample of instances
               of the same workload, one instance per host thread.
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
# HBM bytes (read + written) per stage-2 launch from the rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE runs summarised in profiles/stage2_wave_kernel_cfg5.md, keyed by
# (config, variant); None where not measured.
MEASURED_TRAFFIC = {(5, 0): 6.06e9 + 1.181e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--variant", type=int, default=0, help="stage-2 kernel family (0 auto)")
    ap.add_argument("--no-K", action="store_true", help="do not store back-pointers")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--ext", action="store_true",
                    help="time the extended solver (Appendix B: Algorithms 1, 3, 4 and set "
                         "recovery) on the flag-dependent version of --config (default 3, the "
                         "MobileNetV2-shaped batch) instead of the headline workload")
    ap.add_argument("--graph", action="store_true",
                    help="record the step into a HIP graph once and time its replays")
    ap.add_argument("--fused", action="store_true",
                    help="stage 1 + stage 2 in one launch (dpc_stage12_fused; small instances: "
                         "L <= 63, P <= 2048)")
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
    cfg = inputs.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    T, I, base = inputs.make_batch(cfg, seed=args.seed)
    qi, qt = inputs.budgets(cfg, base)
    Td, Id = torch.from_numpy(T).to(dev), torch.from_numpy(I).to(dev)
    qid, qtd = torch.from_numpy(qi).to(dev), torch.from_numpy(qt).to(dev)
    buf = api.Buffers(cfg.B, cfg.L, cfg.P, len(qi), store_K=not args.no_K)
    api.dpc_set_stage2_variant(args.variant)
    stream = torch.cuda.current_stream()

    if args.fused and not api.dpc_stage12_fused_supported(cfg.L, cfg.P):
        print(f"bench.py --fused: L = {cfg.L}, P = {cfg.P} is outside the single-launch path",
              file=sys.stderr)
        sys.exit(2)

    def step(ev=None):
        if ev:
            ev[0].record(stream)
        if args.fused:
            if ev:
                ev[1].record(stream)         # (stage 1 runs inside the one kernel)
            api.dpc_stage12_fused(Td, Id, buf.Topt, buf.split, buf.M, buf.K)
        else:
            api.dpc_stage1_minplus(Td, buf.Topt, buf.split)
            if ev:
                ev[1].record(stream)
            api.dpc_stage2_knapsack(buf.Topt, Id, buf.M, buf.K, buf.workspace)
        if ev:
            ev[2].record(stream)
        api.dpc_backtrack(buf.Topt, buf.split, Id, buf.M, buf.K, qid, qtd, buf.A, buf.A_len,
                          buf.S, buf.S_len, buf.obj, buf.lat, buf.status)
        if ev:
            ev[3].record(stream)

    for _ in range(args.warmup):
        step()
    api.dpc_stage2_check(buf.workspace)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    if args.graph:
        # (per-stage events are recorded inside the graph once; the replays are timed as a whole)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        stream = torch.cuda.current_stream()
        t0 = time.perf_counter()
        for k in range(args.steps):
            evs[k][0].record(stream)
            graph.replay()
            for x in (1, 2, 3):
                evs[k][x].record(stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(evs[k])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    api.dpc_stage2_check(buf.workspace)

    ms_step = (t1 - t0) * 1e3 / args.steps
    s1 = [e[0].elapsed_time(e[1]) for e in evs]
    s2 = [e[1].elapsed_time(e[2]) for e in evs]
    s3 = [e[2].elapsed_time(e[3]) for e in evs]
    exact = inputs.relax_ops_exact(cfg.B, cfg.L, cfg.P)
    nominal = inputs.relax_ops_nominal(cfg.B, cfg.L, cfg.P)
    s2_avg = float(np.mean(s2))
    ops_per_relax = 2 if args.no_K else 4
    achieved = ops_per_relax * exact / (s2_avg * 1e-3)
    n_ok = int((buf.status == 0).sum().item())

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
                   "queries": int(len(qi)), "store_K": not args.no_K,
                   "stage2_variant": args.variant, "fused_stage12": bool(args.fused),
                   "graph_replay": bool(args.graph),
                   "seed": args.seed},
        "exact_relax_ops_per_s": exact / (ms_step * 1e-3),
        "stage2_exact_relax_ops_per_s": exact / (s2_avg * 1e-3),
        "stage_ms": {"stage1": float(np.mean(s1)), "stage2": s2_avg,
                     "stage2_min": float(np.min(s2)), "backtrack": float(np.mean(s3))},
        "feasible_queries": n_ok,
        "roofline": {
            "bound": "alu", "kernel": "stage 2 (dpc_stage2_knapsack)",
            "achieved": achieved / 1e12, "peak": VALU_PEAK_LANE_OPS / 1e12,
            "unit": "TOP/s", "frac": achieved / VALU_PEAK_LANE_OPS,
            "ops_per_relax": ops_per_relax,
            "traffic": MEASURED_TRAFFIC.get((args.config, args.variant)),
        },
    }

    if not args.no_cpu:
        import oracle
        cores = min(16, os.cpu_count() or 1)
        nb = min(cfg.B, cores)
        # about 10-30 s of CPU work: whole instances, one per thread
        per_inst = inputs.relax_ops_exact(1, cfg.L, cfg.P)
        while nb * per_inst < 2e10 and nb < cfg.B:
            nb += cores
        nb = min(nb, cfg.B)
        sel = qi < nb
        tc0 = time.perf_counter()
        To, sp, Mo, Ko = oracle.solve_batch(T[:nb], I[:nb], cfg.P, want_K=not args.no_K,
                                            threads=cores)
        for b, t in zip(qi[sel], qt[sel]):
            oracle.backtrack(To[b], sp[b], I[b], Mo[b], None if Ko is None else Ko[b], int(t))
        tc1 = time.perf_counter()
        out["cpu_baseline"] = {
            "value": inputs.relax_ops_nominal(nb, cfg.L, cfg.P) / (tc1 - tc0),
            "unit": "relax-ops/s", "cores": min(cores, nb), "kind": "oracle",
            "sample": f"{nb} of {cfg.B} instances of {cfg.name}, all stages, "
                      f"{tc1 - tc0:.2f} s wall",
        }
    print(json.dumps(out))


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
    api.dpc_set_stage2_variant(args.variant)
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
                   "queries": int(len(qi)), "stage2_variant": args.variant, "seed": args.seed},
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
    n_alpha constants -> B instances) + stage 1 + stage 2 + dpc_front + dpc_front_queries +
    dpc_backtrack at every point of every trade-off curve + dpc_chain_latency at A."""
    cid = 3 if args.config == 5 else args.config
    cfg = inputs.CONFIGS[cid]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n_alpha = 16 if cfg.B >= 16 else 1
    T0, I_raw, base, alphas = inputs.make_sweep_batch(cfg, seed=args.seed, n_alpha=n_alpha)
    n_raw = T0.shape[0]
    B = n_raw * n_alpha
    T = np.repeat(T0, n_alpha, axis=0)
    Td = torch.from_numpy(T).to(dev)
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
    api.dpc_set_stage2_variant(args.variant)
    stream = torch.cuda.current_stream()
    names = ["importance_shift", "stage1", "stage2", "front", "front_queries", "backtrack",
             "chain_latency"]

    def step(ev=None):
        calls = [
            lambda: api.dpc_importance_shift(Ird, ald, Id),
            lambda: api.dpc_stage1_minplus(Td, buf.Topt, buf.split),
            lambda: api.dpc_stage2_knapsack(buf.Topt, Id, buf.M, buf.K, buf.workspace),
            lambda: api.dpc_front(buf.M, ft, fo, fl),
            lambda: api.dpc_front_queries(ft, fl, qid, qtd, qn),
            lambda: api.dpc_backtrack(buf.Topt, buf.split, Id, buf.M, buf.K, qid, qtd, buf.A,
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
                   "stage2_variant": args.variant, "seed": args.seed},
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
