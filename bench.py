"""Benchmark of the plan-scoring hot path on one MI355X.

A step is one exhaustive chm_search_best over the whole plan space of the 32-card
configuration (L=48, PP=8, DP=4, M=16, one failed node): unranking, stage sums, memory
filter, 1F1B recurrence per pipeline class, strategy terms and argmin for every partition
of the three strategies and every reroute vector.  The scenario tables are resident in
HBM before the timed region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X VALU: 256 compute units x 4 SIMDs x 32 lanes per clock x 2.4 GHz = 78.6 T int32 lane
# operations per second (the published fp32 vector figure, 157.3 TFLOP/s, is this rate x 2 flops per
# fused multiply-add).  Only simple operations (v_add_u32) issue at that rate; v_max_i32 and
# v_mul_u32_u24, which the path needs, issue at half of it (chm_valu_probe measures both).
ALU_PEAK_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12

# HBM bytes per launch of the config-2 search kernels, per strategy, from the rocprofv3 --pmc runs summarised in
# profiles/search_kernels_config2.md: FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 (KiB; the factors come from the
# 1 GiB calibration copy of the same runs).  Counters cannot be read from inside this process.
CONFIG2_TRAFFIC_BYTES = {0: (178.9 * 2.0 + 4302) * 1024, 1: (133.0 * 2.0 + 510.5) * 1024, 2: (182.2 * 2.0 + 490.6) * 1024}


def algorithmic_ops(fam, feasible):
    """Integer operations the method needs for one search launch of a strategy (not what the kernel
    executes).  Every partition: 3 stage sums per stage and the memory compare per stage.  A
    partition that passes the memory filter in addition: per pipeline class one max and one add
    per recurrence cell (2 x stages x micro-batches cells), 2 Q16 scalings per stage, the
    comm add and the max over pipelines; 4 per stage for the weight-fetch volume; 2 for the cost;
    per stage that lost nodes the products (extra micro-batches x peer stage time) for every count
    0..orphans, one add each, which all reroute vectors share; and per reroute vector the max over
    its peers' products and the compare."""
    S = fam["stages"]
    light = 4 * S
    heavy = sum(4 * n_c * m_c + 2 * n_c + 2 for n_c, m_c in fam["classes"]) + 4 * S + 2
    heavy += sum(R * p + p * t for R, p, t in zip(fam["R"], fam["peers"], fam["orphans"]))
    if fam.get("assign") and fam["strategy"] == 1:
        # least-transfer assignment: the two-index recurrence over (survivor, new stage) pairs, per cell
        # the overlap (min, max, subtract, clamp) and one add and two max
        heavy += sum(7 * n_c * n_c for n_c, _ in fam["classes"])
    return fam["n_part"] * light + feasible * heavy, light, heavy


def copy_calibration():
    """one plain 1 GiB device copy: the known-size reference for scaling FETCH_SIZE / WRITE_SIZE"""
    import torch
    src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def bench_replan(args, note, B, synth):
    """A step = one chm_replan over the 31 surviving nodes of the 32-card shape: every contiguous split of the
    48 layers for every pipeline length the DP range 2..6 produces within 4..12 stages, the least-transfer
    assignment of the 31 nodes per candidate, and the exact ratio objective."""
    import torch
    rp = synth.replan32()
    if args.copy_calibration:
        copy_calibration()
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            B.replan(rp, stream=stream)
            note("warm-up step %d done" % i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        search_ms = assign_ms = 0.0
        for _ in range(args.steps):
            plan, st = B.replan(rp, stream=stream, with_stats=True)
            search_ms += st["search_ms"]
            assign_ms += st["assign_ms"]
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms = wall * 1e3 / args.steps
    search_ms /= args.steps
    assign_ms /= args.steps
    achieved = st["algorithmic_ops"] / (search_ms * 1e-3) / 1e12
    # the same call with bounded split searches (same plan; reported beside the exhaustive figures)
    rb = dict(rp, bounded_search=1)
    with torch.cuda.stream(stream):
        B.replan(rb, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            plan_b, st_b = B.replan(rb, stream=stream, with_stats=True)
        torch.cuda.synchronize()
        ms_b = (time.perf_counter() - t0) * 1e3 / args.steps
    bounded = {"time_to_best_plan_ms": ms_b, "search_kernels_ms": st_b["search_ms"], "splits_evaluated_in_full": st_b["splits_evaluated"],
               "same_plan_as_exhaustive": bool(plan_b == plan)}
    note("bounded re-planning: %s" % bounded)
    out = {"metric": "candidate plans scored/sec + time-to-best-plan per failure event (1 GPU)",
           "value": st["splits_scored"] / (ms * 1e-3), "unit": "plans/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "int32", "data": "synthetic",
           "config": {"workload": "replan32: L=48, 31 of 32 nodes survive, DP 2..6, PP 4..12, 64 micro-batches per step; "
                                  "every contiguous split per pipeline length", "splits_scored_per_step": st["splits_scored"],
                      "splits_feasible": st["splits_feasible"], "candidates": plan["n_candidates"]},
           "time_to_best_plan_ms": ms, "search_kernels_ms": search_ms, "assignment_kernels_ms": assign_ms,
           "bounded_search": bounded, "best": plan,
           "roofline": {"bound": "alu", "kernel": "split search (all pipeline lengths)", "achieved": achieved,
                        "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / ALU_PEAK_TOPS, "traffic": None,
                        "algorithmic_ops_per_launch": st["algorithmic_ops"]}}
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        # the oracle's exhaustive split of the shortest pipeline length of the candidates (a bounded sample)
        n, M = 6, 12
        t0 = time.perf_counter()
        O.best_split(rp["fwd_us"], rp["bwd_us"], rp["mem_mib"], None, n, M, rp["mem_cap_mib"])
        t = time.perf_counter() - t0
        n_splits = O.binom(rp["L"] - 1, n - 1)
        out["cpu_baseline"] = {"value": n_splits / t, "unit": "plans/s", "cores": 1, "kind": "oracle",
                               "sample": "oracle best split over all %d splits into %d stages, %d micro-batches (%.1f s)" % (n_splits, n, M, t)}
    print(json.dumps(out))


def bench_score(args, note, B, synth):
    """A step = chm_score_plans over three windows of 2^27 consecutive plan indices of config 2, one inside
    every strategy's index range: the cost of every plan index is stored (8 bytes per plan), so this
    is the one part of the path that is bound by HBM writes."""
    import torch
    g = B.Scenario(synth.config2())
    n = 1 << 27
    out = torch.empty(n, dtype=torch.int64, device="cuda")
    if args.copy_calibration:
        copy_calibration()
    firsts = [f["offset"] + min(f["n_part"] * f["n_reroute"] - n, (f["n_part"] * f["n_reroute"]) // 3) for f in g.families]
    firsts = [max(f["offset"], x) for f, x in zip(g.families, firsts)]
    counts = [min(n, f["n_part"] * f["n_reroute"]) for f in g.families]
    stream = torch.cuda.Stream()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(firsts) + 1)]
    ms = [0.0] * len(firsts)
    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            for first, cnt in zip(firsts, counts):
                g.score_plans(first, cnt, out=out, stream=stream)
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            ev[0].record(stream)
            for k, (first, cnt) in enumerate(zip(firsts, counts)):
                g.score_plans(first, cnt, out=out, stream=stream)
                ev[k + 1].record(stream)
            stream.synchronize()
            for k in range(len(firsts)):
                ms[k] += ev[k].elapsed_time(ev[k + 1])
        wall = time.perf_counter() - t0
    ms = [m / args.steps for m in ms]
    total = sum(counts)
    # the window of the rerouting strategy is the one bound by the stores (a few operations per plan index, the
    # partition's recurrence is shared by its reroute vectors); the other two run one recurrence per stored cost
    # and are bound by it like the search (see kernel_ms_per_strategy of the search workloads)
    store_bound = [k for k, f in enumerate(g.families) if f["n_reroute"] > 1]
    dom = store_bound[0] if store_bound else max(range(len(ms)), key=lambda k: ms[k])
    gbs = [8.0 * c / (m * 1e-3) / 1e9 for c, m in zip(counts, ms)]
    out_json = {"metric": "candidate plans scored/sec + time-to-best-plan per failure event (1 GPU)",
                "value": total / (wall / args.steps), "unit": "plans/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
                "dtype": "int32", "data": "synthetic",
                "config": {"workload": "score2: chm_score_plans over 2^27 consecutive plan indices inside each strategy of config 2",
                           "plan_indices_per_step": total, "windows": [{"strategy": f["strategy"], "first": x, "count": c}
                                                                      for f, x, c in zip(g.families, firsts, counts)]},
                "ms_per_strategy": ms, "store_gb_per_s_per_strategy": gbs,
                "roofline": {"bound": "hbm", "kernel": "cost store, strategy %d" % g.families[dom]["strategy"], "achieved": gbs[dom],
                             "peak": 8000.0, "unit": "GB/s", "frac": gbs[dom] / 8000.0, "traffic": None,
                             "algorithmic_bytes_per_launch": 8.0 * counts[dom]}}
    print(json.dumps(out_json))


def bench_lists(args, note, B, synth):
    """config 4: 2^24 seeded random partitions per strategy (L=96, PP=16, DP=2, M=64, one failure, cap chosen
    for about 30 % infeasible plans).  A step = one chm_search_cuts per strategy over its list of cut
    positions, with the cost of every entry stored."""
    import numpy as np
    import torch
    sc = synth.config4(mem_cap_mib=synth.CONFIG4_CAP_30PCT)
    g = B.Scenario(sc)
    n, chunk = 1 << 24, 1 << 20
    lists = {}
    for f in g.families:
        k = f["stages"] - 1
        d_cuts = torch.empty((n, k), dtype=torch.uint8, device="cuda")
        for c0 in range(0, n, chunk):
            cuts = synth.random_partitions(synth.BASE_SEED + 4, 1000 * f["strategy"] + c0 // chunk, chunk, sc["L"], k)
            d_cuts[c0:c0 + chunk] = torch.from_numpy(cuts).cuda()
        lists[f["strategy"]] = d_cuts
        note("strategy %d: %d partitions ready" % (f["strategy"], n))
    costs = torch.empty(n, dtype=torch.int64, device="cuda")
    stream = torch.cuda.Stream()
    g.set_timing(True)
    fam_ms = np.zeros(3)
    feasible = np.zeros(3)
    with torch.cuda.stream(stream):
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            for st, d_cuts in lists.items():
                g.search_cuts(st, d_cuts, costs=costs, stream=stream)
        stream.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            for st, d_cuts in lists.items():
                rc, best, pos = g.search_cuts(st, d_cuts, costs=costs, stream=stream)
                tm = g.get_timing()
                fam_ms[st] += tm["family_ms"][st]
                feasible[st] = tm["feasible"][st]
        stream.synchronize()
        wall = time.perf_counter() - t0
    fam_ms /= args.steps
    ms = wall * 1e3 / args.steps
    # the same argmin per list without the cost store, exhaustive and bounded (reported beside `value`)
    winners, modes = {}, {}
    with torch.cuda.stream(stream):
        for mode in (0, 1):
            g.set_bounded_search(mode)
            for st, d_cuts in lists.items():
                g.search_cuts(st, d_cuts, stream=stream)
            stream.synchronize()
            t0 = time.perf_counter()
            evaluated = np.zeros(3)
            for _ in range(args.steps):
                for st, d_cuts in lists.items():
                    rc_m, best_m, pos_m = g.search_cuts(st, d_cuts, stream=stream)
                    winners.setdefault(st, []).append((rc_m, pos_m, best_m["cost"]))
                    evaluated[st] = g.get_timing()["feasible"][st]
            stream.synchronize()
            modes[mode] = {"ms_per_step": (time.perf_counter() - t0) * 1e3 / args.steps, "entries_evaluated": [float(x) for x in evaluated]}
        g.set_bounded_search(0)
    bounded = {"argmin_only_ms_per_step": modes[0]["ms_per_step"], "bounded_ms_per_step": modes[1]["ms_per_step"],
               "entries_evaluated_exhaustive": modes[0]["entries_evaluated"], "entries_evaluated_bounded": modes[1]["entries_evaluated"],
               "same_winners": all(len(set(v)) == 1 for v in winners.values())}
    note("list search without cost store: %s" % bounded)
    ops = np.zeros(3)
    for f in g.families:
        fam = dict(f, classes=g.family_classes(f["strategy"]), n_part=n, assign=0,
                   peers=[p for p, _ in g.reroute_shape()] if f["strategy"] == 2 else [],
                   R=[r for _, r in g.reroute_shape()] if f["strategy"] == 2 else [],
                   orphans=[sc["M"]] if f["strategy"] == 2 else [])
        ops[f["strategy"]] = algorithmic_ops(fam, feasible[f["strategy"]])[0]
    dom = int(np.argmax(fam_ms))
    achieved = ops[dom] / (fam_ms[dom] * 1e-3) / 1e12
    evals = sum(n * (sum(r for _, r in g.reroute_shape()) if f["strategy"] == 2 else 1) for f in g.families)
    print(json.dumps({"metric": "candidate plans scored/sec + time-to-best-plan per failure event (1 GPU)",
                      "value": evals / (ms * 1e-3), "unit": "plans/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32",
                      "data": "synthetic",
                      "config": {"workload": "config4: L=96 PP=16 DP=2 M=64, 1 failed node, 2^24 random partitions per strategy "
                                             "(explicit lists), cap %d MiB" % sc["mem_cap_mib"],
                                 "partitions_per_strategy": n, "plans_scored_per_step": evals, "failed_nodes": sc["failed_nodes"]},
                      "kernel_ms_per_strategy": [float(x) for x in fam_ms], "bounded_search": bounded,
                      "feasible_partitions_per_strategy": [float(x) for x in feasible],
                      "roofline": {"bound": "alu", "kernel": "list search, strategy %d" % dom, "achieved": achieved,
                                   "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / ALU_PEAK_TOPS, "traffic": None,
                                   "algorithmic_ops_per_launch": float(ops[dom])}}))



def threaded_sweep(B, handles, plans, n_threads=4, reps=3):
    """one search per handle, the handles dealt out to n_threads host threads with a stream each (independent
    handles may be used concurrently); returns (median ms for all handles, every plan equals `plans`)"""
    import threading
    import numpy as np
    import torch

    def sweep(t, out):
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            for i in range(t, len(handles), n_threads):
                out[i] = handles[i].search_best(7, stream=st)[1]

    times, same = [], True
    for _ in range(reps):
        found = [None] * len(handles)
        threads = [threading.Thread(target=sweep, args=(t, found)) for t in range(n_threads)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for th in threads:
            th.start()
        for th in threads:
            th.join()
        times.append((time.perf_counter() - t0) * 1e3)
        same = same and all(a is not None and a["index"] == b[1]["index"] and a["cost"] == b[1]["cost"]
                            for a, b in zip(found, plans))
    return float(np.median(times)), same


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--ttb-runs", type=int, default=10)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2", "config3", "config4", "config5", "replan32", "score2"],
                    help="config2 (the 32-card shape) is the benchmark; the others are for profiling; replan32 times "
                         "chm_replan (search over DP/PP degrees) for the 31 nodes that survive in config2")
    ap.add_argument("--transfer-assign", type=int, default=0, choices=[0, 1],
                    help="1: the re-partition strategy counts the weights to fetch under the least-transfer "
                         "assignment of survivors to new stages (default 0: survivors in stage order)")
    ap.add_argument("--plan-cache", default=None,
                    help="write the best plan of every scenario of the workload to this file, one JSON object per "
                         "line (the cache of pre-computed plans the Planner keeps for possible failures)")
    ap.add_argument("--filter-compaction", type=int, default=-1, choices=[-1, 0, 1],
                    help="chm_set_filter_compaction mode of the search workloads: -1 chosen by the library per strategy, 0 off, 1 on")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size reference for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the plan search runs on a single MI355X and nothing here shards "
              "across devices; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    def note(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    import numpy as np
    import torch
    from paper_2508_21613_amd import binding as B
    from paper_2508_21613_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    if args.workload == "replan32":
        return bench_replan(args, note, B, synth)
    if args.workload == "score2":
        return bench_score(args, note, B, synth)
    if args.workload == "config4":
        return bench_lists(args, note, B, synth)
    workloads = {
        "config1": ("config1: L=32 PP=4 DP=2 M=8, 1 failed node", lambda: [synth.config1()]),
        "config2": ("config2: L=48 PP=8 DP=4 M=16, 1 failed node", lambda: [synth.config2()]),
        "config3": ("config3: L=40 PP=4 DP=8 M=32, 2 failed nodes, Q16 speed factors, reroute cap 16", lambda: [synth.config3()]),
        "config5": ("config5: L=40 PP=8 DP=4 M=16, all 32 single and 496 double node failures",
                    lambda: [synth.config5(fs) for fs in synth.config5_failure_sets()]),
    }
    label, make = workloads[args.workload]
    scenarios = [dict(sc, transfer_assign=args.transfer_assign) for sc in make()]
    if args.transfer_assign:
        label += ", least-transfer assignment"
    t0 = time.perf_counter()
    handles = [B.Scenario(sc) for sc in scenarios]
    load_ms = (time.perf_counter() - t0) * 1e3
    note("%d scenario(s) loaded in %.1f ms" % (len(handles), load_ms))
    stream = torch.cuda.Stream()

    def family_work(g, sc):
        shape = g.reroute_shape()
        lost = {}
        for node in sc["failed_nodes"]:
            lost[node % sc["PP"]] = lost.get(node % sc["PP"], 0) + 1
        orphans = [lost[s] * sc["M"] for s in sorted(lost)]     # per stage that lost nodes, ascending
        fams = []
        for f in g.families:
            d = dict(f)
            d["orphans"] = orphans if f["strategy"] == 2 else []
            d["classes"] = g.family_classes(f["strategy"])
            d["peers"] = [p for p, _ in shape] if f["strategy"] == 2 else []
            d["R"] = [r for _, r in shape] if f["strategy"] == 2 else []
            d["assign"] = args.transfer_assign
            fams.append(d)
        return fams

    work = [family_work(g, sc) for g, sc in zip(handles, scenarios)]
    fit_share = [g.set_filter_compaction(args.filter_compaction) for g in handles][0]

    if args.copy_calibration:
        copy_calibration()
    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            for g in handles:
                g.search_best(7, stream=stream)
            note("warm-up step %d done" % i)
        for g in handles:
            g.set_timing(True)
        fam_ms = np.zeros(3)
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        plans = [None] * len(handles)
        for _ in range(args.steps):
            for i, g in enumerate(handles):
                rc, best = g.search_best(7, stream=stream)
                plans[i] = (rc, best)
                fam_ms += np.array(g.get_timing()["family_ms"])
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    fam_ms /= args.steps
    if args.plan_cache:
        with open(args.plan_cache, "w") as fh:
            for sc_i, (rc_i, best_i) in zip(scenarios, plans):
                fh.write(json.dumps({"failed_nodes": sc_i["failed_nodes"], "rc": rc_i, "index": best_i["index"], "cost": best_i["cost"],
                                     "strategy": best_i["strategy"], "cuts": best_i["cuts"],
                                     "reroute": best_i["reroute"] if best_i["strategy"] == 2 else None}) + "\n")
        note("best plan of %d scenario(s) written to %s" % (len(plans), args.plan_cache))
    note("timed %d steps: %.3f ms per step, kernel ms per strategy %s" % (args.steps, ms_per_step, fam_ms))

    # work done per step, from the library's own counters of the last search on every handle
    evaluations = np.zeros(3)
    feasible = np.zeros(3)
    ops = np.zeros(3)
    n_part_total, cells, plan_indices = 0, 0, 0
    for g, fams in zip(handles, work):
        tm = g.get_timing()
        evaluations += np.array(tm["evaluations"], dtype=float)
        feasible += np.array(tm["feasible"], dtype=float)
        plan_indices += g.n_plans
        for f in fams:
            ops[f["strategy"]] += algorithmic_ops(f, tm["feasible"][f["strategy"]])[0]
            n_part_total += f["n_part"]
            cells += f["n_part"] * sum(2 * n * m for n, m in f["classes"])
    n_plans = float(evaluations.sum())

    # time-to-best-plan: load + search on a fresh handle, median over --ttb-runs (first scenario)
    ttb = []
    for _ in range(args.ttb_runs):
        t0 = time.perf_counter()
        g2 = B.Scenario(scenarios[0])
        g2.search_best(7, stream=stream)
        ttb.append((time.perf_counter() - t0) * 1e3)
        g2.close()
    ttb_ms = float(np.median(ttb)) if ttb else None
    note("time to best plan (load + search): %s ms" % ttb_ms)

    # many scenarios: the host side of a call (launches, one synchronisation) hides behind other threads' kernels
    threaded_exhaustive = None
    if args.ttb_runs and len(handles) >= 8:
        ms_t, same_t = threaded_sweep(B, handles, plans, reps=2)
        threaded_exhaustive = {"search_ms_all_scenarios_4_threads": ms_t, "same_plans": bool(same_t)}
        note("exhaustive search from four host threads: %s" % threaded_exhaustive)

    # the same with chm_set_bounded_search: same plan, most partitions skipped by a lower bound of their cost.
    # Reported beside the exhaustive figures, never inside `value` (which counts plans that were scored).
    bounded = None
    if args.ttb_runs:
        ttb_b, search_b, same = [], [], True
        for g in handles:
            g.set_bounded_search(True)
        for _ in range(args.ttb_runs):
            t0 = time.perf_counter()
            g2 = B.Scenario(scenarios[0])
            g2.set_bounded_search(True)
            rc_b, best_b = g2.search_best(7, stream=stream)
            ttb_b.append((time.perf_counter() - t0) * 1e3)
            g2.close()
            same = same and (rc_b, best_b["index"], best_b["cost"]) == (plans[0][0], plans[0][1]["index"], plans[0][1]["cost"])
            t0 = time.perf_counter()
            swept = [g.search_best(7, stream=stream)[1] for g in handles]
            search_b.append((time.perf_counter() - t0) * 1e3)
            same = same and all(a["index"] == b[1]["index"] and a["cost"] == b[1]["cost"] for a, b in zip(swept, plans))
        ev = np.zeros(3)
        for g in handles:
            ev += np.array(g.get_timing()["evaluated"], dtype=float)
        # a bounded search is bound by launch and synchronisation latency, not by the GPU: independent scenarios
        # searched from four host threads (a stream each) overlap
        threaded_ms = None
        if len(handles) >= 8:
            threaded_ms, same_t = threaded_sweep(B, handles, plans)
            same = same and same_t
        for g in handles:
            g.set_bounded_search(False)
        bounded = {"time_to_best_plan_ms": float(np.median(ttb_b)), "search_ms_all_scenarios": float(np.median(search_b)),
                   "search_ms_all_scenarios_4_threads": threaded_ms,
                   "partitions_evaluated_in_full": [float(x) for x in ev], "same_plans_as_exhaustive": bool(same)}
        note("bounded search: %s" % bounded)

    # roofline of the dominant kernel
    dom = int(np.argmax(fam_ms))
    achieved = ops[dom] / (fam_ms[dom] * 1e-3) / 1e12
    fam0 = [f for f in work[0] if f["strategy"] == dom]
    _, ops_light, ops_heavy = algorithmic_ops(fam0[0], 0) if fam0 else (0, 0, 0)

    probes = {name: B.valu_probe(kind, 3000, stream=stream) / 1e12
              for kind, name in ((0, "v_add_u32"), (1, "v_max_i32"), (2, "max_add_cell_chain"))}
    note("measured VALU rates (T lane-ops/s): %s" % probes)
    sc = scenarios[0]
    out = {
        "metric": "candidate plans scored/sec + time-to-best-plan per failure event (1 GPU)",
        "value": n_plans / (ms_per_step * 1e-3),
        "unit": "plans/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": label + ", exhaustive search over all strategies",
                   "scenarios": len(handles), "plans_scored_per_step": n_plans, "plan_indices": plan_indices,
                   "partitions": n_part_total, "failed_nodes": sc["failed_nodes"] if len(handles) == 1 else "all",
                   "families": [{k: f[k] for k in ("strategy", "stages", "n_part", "n_reroute")} for f in work[0]]},
        "time_to_best_plan_ms": ttb_ms, "load_ms": load_ms,
        "time_to_best_plan_bounded_ms": bounded["time_to_best_plan_ms"] if bounded else None,
        "bounded_search": bounded,
        "exhaustive_search_4_threads": threaded_exhaustive,
        "partition_evals_per_s": n_part_total / (ms_per_step * 1e-3),
        "recurrence_cells_per_s": cells / (ms_per_step * 1e-3),
        "kernel_ms_per_strategy": [float(x) for x in fam_ms],
        "best": {"index": best["index"], "cost": best["cost"], "strategy": best["strategy"], "cuts": best["cuts"]},
        "roofline": {"bound": "alu", "kernel": "search, strategy %d" % dom, "achieved": achieved,
                     "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / ALU_PEAK_TOPS,
                     "measured_valu_rates_tops": probes,
                     "frac_of_measured_cell_rate": achieved / probes["max_add_cell_chain"],
                     "traffic": CONFIG2_TRAFFIC_BYTES[dom] if args.workload == "config2" and not args.transfer_assign else None,
                     "kernel_ms": float(fam_ms[dom]), "algorithmic_ops_per_launch": float(ops[dom]),
                     "feasible_partitions": float(feasible[dom]),
                     "algorithmic_ops_per_feasible_partition": ops_light + ops_heavy,
                     "algorithmic_ops_per_infeasible_partition": ops_light},
        "feasible_partitions_per_strategy": [float(x) for x in feasible],
        "filter_compaction": {"mode": args.filter_compaction, "sampled_fit_share": fit_share},
    }

    if not args.no_cpu_baseline:
        from oracle import oracle as O
        o = O.Scenario(scenarios[0])
        spent = 0.0
        per_family = []
        for f in o.families:               # the same three strategies, a slice from the middle of each rank space
            share = max(0.1, (f["n_part"] * f["n_reroute"]) / o.n_plans * 0.8)
            budget = args.cpu_seconds * share
            mid = f["n_part"] // 2
            n0 = min(500, f["n_part"] - mid)
            t0 = time.perf_counter()
            o.search_range(f["strategy"], mid, n0)
            t_cal = max(time.perf_counter() - t0, 1e-4)
            n = int(max(n0, min(f["n_part"] - mid, budget * n0 / t_cal)))
            t0 = time.perf_counter()
            _, _, ev = o.search_range(f["strategy"], mid, n)
            t = time.perf_counter() - t0
            per_family.append((f["strategy"], n, ev, t))
            note("oracle: strategy %d, %d partitions in %.2f s" % (f["strategy"], n, t))
            spent += t + t_cal
        # whole-job rate of the oracle: time it would need for the full space at these per-family rates
        full_s = sum(t * (o.family(s)["n_part"] / n) for s, n, ev, t in per_family)
        o_plans = sum(f["n_part"] * (sum(r for _, r in handles[0].reroute_shape()) if f["strategy"] == 2 and handles[0].reroute_shape() else 1)
                      for f in o.families)
        out["cpu_baseline"] = {"value": o_plans / full_s, "unit": "plans/s", "cores": 1, "kind": "oracle",
                               "sample": "oracle search over %s partitions from the middle of the rank space of strategies %s (%.1f s of CPU work), "
                                         "extrapolated per strategy to the full space" %
                                         ([n for _, n, _, _ in per_family], [s for s, _, _, _ in per_family], spent),
                               "full_space_seconds_estimate": full_s}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
