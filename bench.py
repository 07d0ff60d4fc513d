"""Benchmark of the plan-scoring hot path on one MI355X.

A step is one exhaustive chm_search_best over the whole plan space of the 32-card
configuration (L=48, PP=8, DP=4, M=16, one failed node): unranking, stage sums, memory
filter, 1F1B recurrence per pipeline class, strategy terms and argmin for every partition
of the three strategies and every reroute vector.  The scenario tables are resident in
HBM before the timed region.  Prints one JSON line; with no flags that line also carries a
`workloads` block with the other configurations (1, 3, 4, 5), the cost store and the
re-planning search at a few steps each.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "candidate plans scored/sec + time-to-best-plan per failure event (1 GPU)"

# MI355X VALU: 256 compute units x 4 SIMDs x 32 lanes per clock x 2.4 GHz = 78.6 T int32 lane
# operations per second (the published fp32 vector figure, 157.3 TFLOP/s, is this rate x 2 flops per
# fused multiply-add).  Only simple operations (v_add_u32) issue at that rate; v_max_i32 and
# v_mul_u32_u24, which the path needs, issue at half of it (chm_valu_probe measures both).
ALU_PEAK_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12

# From the rocprofv3 --pmc runs summarised in profiles/search_kernels_config2.md (counters cannot be read from
# inside this process), per strategy kernel of config 2:
# HBM bytes per launch = FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB (factors from the 1 GiB calibration copy of the same runs)
CONFIG2_TRAFFIC_BYTES = {0: (163.9 * 2.0 + 447.6) * 1024, 1: (125.0 * 2.0 + 256.4) * 1024, 2: (186.6 * 2.0 + 475.4) * 1024}
# executed VALU lane-instructions per partition = SQ_INSTS_VALU x 64 / partitions of the family
CONFIG2_EXECUTED_LANE_INSTR_PER_PARTITION = {0: 558.0, 1: 419.0, 2: 754.0}


def note(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


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


def shared_prefix_ops(peers, total, cap):
    """Operations of one partition's reroute sweep of one stage in the formulation the large-space sweep kernel uses
    (the vectors of a group share the largest product of their first peers - 3 entries; per value of the entry before
    the last two one add, two max and one min; the least larger-product of the last two entries per remaining sum
    from a table built once, one max and one min per pair): the count that kernel's executed instructions are close to."""
    cap = min(cap, total) if cap > 0 else total
    q = peers - 3
    if q < 0:
        return None
    # number of ways to fill the first q entries (each 0..cap) with a given sum
    ways = [1] + [0] * total
    for _ in range(q):
        ways = [sum(ways[t - v] for v in range(0, min(cap, t) + 1)) for t in range(total + 1)]
    groups = runs = 0
    for used, w in enumerate(ways):
        rest = total - used                                   # for the last three entries
        lo, hi = max(0, rest - 2 * cap), min(cap, rest)
        if w and lo <= hi:
            groups += w
            runs += w * (hi - lo + 1)
    pairs = sum(min(cap, r) - max(0, r - cap) + 1 for r in range(2 * cap + 1))
    return groups * max(0, 2 * q - 1) + runs * 4 + pairs * 2 + 2 * cap


def copy_calibration():
    """one plain 1 GiB device copy: the known-size reference for scaling FETCH_SIZE / WRITE_SIZE"""
    import torch
    src = torch.zeros(1 << 28, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def host_cores():
    """cores this process may run on (the GPU machine gives a one-GPU job a share of the host)"""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit():
        n = min(n, max(1, int(env)))
    return n


def oracle_all_cores(scenario, seconds, cores):
    """The oracle searching slices from the middle of every strategy's rank space, as independent single-threaded
    workers on `cores` host threads (one handle each; the C calls release the interpreter lock), about `seconds`
    of wall clock.  Returns per-strategy (partitions done by all workers, evaluations, wall seconds) and the
    seconds the oracle alone (one thread) would need for the whole space at the measured per-core rates."""
    from concurrent.futures import ThreadPoolExecutor
    from oracle import oracle as O
    probe = O.Scenario(scenario)
    fams = probe.families
    weights = []
    for f in fams:                                   # calibration: time per partition of every strategy, one thread
        mid = f["n_part"] // 2
        n0 = 1
        while True:
            n0 = max(1, min(n0, f["n_part"] - mid))
            t0 = time.perf_counter()
            probe.search_range(f["strategy"], mid, n0)
            dt = time.perf_counter() - t0
            if dt >= 0.05 or n0 >= 256 or n0 >= f["n_part"] - mid:
                break
            n0 *= 4
        weights.append(max(dt, 1e-5) / n0)
    total_cost = sum(w * f["n_part"] for w, f in zip(weights, fams))
    rows = []
    for f, w in zip(fams, weights):
        share = max(0.1, w * f["n_part"] / total_cost * 0.8)
        per_worker = int(max(1, min(f["n_part"] // (2 * cores) or 1, seconds * share / w)))
        mid = f["n_part"] // 2
        first = max(0, mid - per_worker * cores // 2)

        def work(i, f=f, first=first, per_worker=per_worker):
            o = O.Scenario(scenario)
            lo = min(first + i * per_worker, f["n_part"] - 1)
            n = min(per_worker, f["n_part"] - lo)
            _, _, ev = o.search_range(f["strategy"], lo, n)
            o.close()
            return n, ev

        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as pool:
            got = list(pool.map(work, range(cores)))
        wall = time.perf_counter() - t0
        rows.append({"strategy": f["strategy"], "partitions": sum(n for n, _ in got), "evaluations": sum(e for _, e in got),
                     "wall_s": wall, "n_part": f["n_part"], "n_reroute_evals": got[0][1] / max(1, got[0][0])})
        note("oracle: strategy %d, %d partitions on %d cores in %.2f s" % (f["strategy"], rows[-1]["partitions"], cores, wall))
    probe.close()
    return rows


def cpu_baseline_record(scenario, seconds, what):
    cores = host_cores()
    rows = oracle_all_cores(scenario, seconds, cores)
    # aggregate: all cores busy; per core: the same work divided by the workers
    full_wall_s = sum(r["wall_s"] * r["n_part"] / r["partitions"] for r in rows)
    plans = sum(r["n_part"] * r["n_reroute_evals"] for r in rows)
    return {"value": plans / full_wall_s, "unit": "plans/s", "cores": cores, "kind": "oracle",
            "per_core_value": plans / (full_wall_s * cores), "host_cores_available": os.cpu_count(),
            "extrapolated": True,
            "sample": "%s: oracle exhaustive search over %s partitions from the middle of the rank space of strategies %s, "
                      "split over %d independent single-threaded workers (%.1f s of wall clock), extrapolated per strategy "
                      "to the full space" % (what, [r["partitions"] for r in rows], [r["strategy"] for r in rows], cores,
                                              sum(r["wall_s"] for r in rows)),
            "full_space_seconds_estimate_all_cores": full_wall_s,
            "full_space_core_seconds_estimate": full_wall_s * cores}


# ---------------------------------------------------------------------------------------------------------
# re-planning over DP/PP degrees
# ---------------------------------------------------------------------------------------------------------
def bench_replan(args, B, synth):
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
    # the cached plans for the loss of 1 .. 3 nodes (chm_replan_table) against three calls of chm_replan
    order = dict(rp, failed_nodes=list(rp["failed_nodes"]) + [13, 20])
    with torch.cuda.stream(stream):
        B.replan_table(order, 3, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        table = B.replan_table(order, 3, stream=stream)
        t_table = (time.perf_counter() - t0) * 1e3
        t0 = time.perf_counter()
        single = [B.replan(dict(order, failed_nodes=order["failed_nodes"][:n]), stream=stream) for n in (1, 2, 3)]
        t_single = (time.perf_counter() - t0) * 1e3
    table_rec = {"failure_order": order["failed_nodes"], "table_ms": t_table, "entry_by_entry_ms": t_single, "same_plans": bool(table == single),
                 "dp_per_entry": [p.get("dp") for p in table]}
    note("re-plan table for the loss of 1..3 nodes: %s" % table_rec)
    out = {"metric": METRIC,
           "value": st["splits_scored"] / (ms * 1e-3), "unit": "plans/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "int32", "data": "synthetic",
           "config": {"workload": "replan32: L=48, 31 of 32 nodes survive, DP 2..6, PP 4..12, 64 micro-batches per step; "
                                  "every contiguous split per pipeline length", "splits_scored_per_step": st["splits_scored"],
                      "splits_feasible": st["splits_feasible"], "candidates": plan["n_candidates"]},
           "time_to_best_plan_ms": ms, "search_kernels_ms": search_ms, "assignment_kernels_ms": assign_ms,
           "bounded_search": bounded, "replan_table_1_to_3": table_rec, "best": plan,
           "roofline": {"bound": "alu", "kernel": "split search (all pipeline lengths)", "achieved": achieved,
                        "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / ALU_PEAK_TOPS, "traffic": None,
                        "kernel_ms": search_ms, "algorithmic_ops_per_launch": st["algorithmic_ops"]}}
    if not args.no_cpu_baseline:
        from oracle import oracle as O
        # the oracle's exhaustive split of the shortest pipeline length of the candidates (a bounded sample)
        n, M = 6, 12
        t0 = time.perf_counter()
        O.best_split(rp["fwd_us"], rp["bwd_us"], rp["mem_mib"], None, n, M, rp["mem_cap_mib"])
        t = time.perf_counter() - t0
        n_splits = O.binom(rp["L"] - 1, n - 1)
        out["cpu_baseline"] = {"value": n_splits / t, "unit": "plans/s", "cores": 1, "kind": "oracle",
                               "host_cores_available": os.cpu_count(),
                               "sample": "oracle best split over all %d splits into %d stages, %d micro-batches (%.1f s, one thread)" % (n_splits, n, M, t)}
    return out


# ---------------------------------------------------------------------------------------------------------
# cost store
# ---------------------------------------------------------------------------------------------------------
def bench_score(args, B, synth):
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
    g.close()
    return {"metric": METRIC,
            "value": total / (wall / args.steps), "unit": "plans/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": wall * 1e3 / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "int32", "data": "synthetic",
            "config": {"workload": "score2: chm_score_plans over 2^27 consecutive plan indices inside each strategy of config 2",
                       "plan_indices_per_step": total, "windows": [{"strategy": f["strategy"], "first": x, "count": c}
                                                                  for f, x, c in zip(g.families, firsts, counts)]},
            "ms_per_strategy": ms, "store_gb_per_s_per_strategy": gbs,
            "roofline": {"bound": "hbm", "kernel": "cost store, strategy %d" % g.families[dom]["strategy"], "achieved": gbs[dom],
                         "peak": 8000.0, "unit": "GB/s", "frac": gbs[dom] / 8000.0, "traffic": None, "kernel_ms": ms[dom],
                         "algorithmic_bytes_per_launch": 8.0 * counts[dom]}}


# ---------------------------------------------------------------------------------------------------------
# explicit lists (config 4)
# ---------------------------------------------------------------------------------------------------------
def random_partitions_device(synth, seed, stream, n, L, k):
    """synth.random_partitions computed on the GPU with torch (same generator, same values): n rows of k distinct
    cut positions of 1..L-1, ascending, as a uint8 CUDA tensor.  The 64-bit mix runs in wrapping int64 arithmetic;
    the logical right shifts are masked and the keys are compared as unsigned (sign bit flipped)."""
    import torch

    def c(v):                                    # a 64-bit constant as a (wrapped) int64
        v &= (1 << 64) - 1
        return v - (1 << 64) if v >= (1 << 63) else v

    def shr(z, b):                               # logical shift right of the 64-bit pattern
        return (z >> b) & ((1 << (64 - b)) - 1)

    m = n * (L - 1)
    i = torch.arange(1, m + 1, dtype=torch.int64, device="cuda")
    base = c((seed & ((1 << 64) - 1)) * 0x9E3779B97F4A7C15 + (stream & ((1 << 64) - 1)) * 0xD1B54A32D192ED03)
    z = i * c(0x8CB92BA72F3D8DD7) + base
    z = (z ^ shr(z, 30)) * c(0xBF58476D1CE4E5B9)
    z = (z ^ shr(z, 27)) * c(0x94D049BB133111EB)
    z = z ^ shr(z, 31)
    keys = (z ^ c(1 << 63)).view(n, L - 1)       # unsigned order as signed order
    order = torch.argsort(keys, dim=1, stable=True)[:, :k]
    return (torch.sort(order, dim=1).values + 1).to(torch.uint8)


def bench_lists(args, B, synth):
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
            d_cuts[c0:c0 + chunk] = random_partitions_device(synth, synth.BASE_SEED + 4, 1000 * f["strategy"] + c0 // chunk, chunk, sc["L"], k)
        # the generator on the device gives the very lists of the seeded host generator (checked on a few rows)
        check = synth.random_partitions(synth.BASE_SEED + 4, 1000 * f["strategy"], 512, sc["L"], k)
        assert (d_cuts[:512].cpu().numpy() == check).all(), "device and host list generators differ"
        lists[f["strategy"]] = d_cuts
        note("config4 strategy %d: %d partitions ready" % (f["strategy"], n))
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
    out = {"metric": METRIC,
           "value": evals / (ms * 1e-3), "unit": "plans/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int32",
           "data": "synthetic",
           "config": {"workload": "config4: L=96 PP=16 DP=2 M=64, 1 failed node, 2^24 random partitions per strategy "
                                  "(explicit lists), cap %d MiB" % sc["mem_cap_mib"],
                      "partitions_per_strategy": n, "plans_scored_per_step": evals, "failed_nodes": sc["failed_nodes"]},
           "time_to_best_plan_ms": ms, "partition_evals_per_s": 3 * n / (ms * 1e-3),
           "kernel_ms_per_strategy": [float(x) for x in fam_ms], "bounded_search": bounded,
           "feasible_partitions_per_strategy": [float(x) for x in feasible],
           "roofline": {"bound": "alu", "kernel": "list search, strategy %d" % dom, "achieved": achieved,
                        "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / ALU_PEAK_TOPS, "traffic": None,
                        "kernel_ms": float(fam_ms[dom]), "algorithmic_ops_per_launch": float(ops[dom])}}
    if not args.no_cpu_baseline:
        # the oracle scoring the first entries of every list, on all cores
        from concurrent.futures import ThreadPoolExecutor
        from oracle import oracle as O
        cores = host_cores()
        per = 2000
        t_all, n_all = 0.0, 0
        for f in g.families:
            if f["n_reroute"] != 1:
                continue
            ranks = O.partition_rank_batch(lists[f["strategy"]][:per * cores].cpu().numpy())

            def work(i, f=f, ranks=ranks):
                o = O.Scenario(sc)
                o.score_ranks(f["strategy"], ranks[i * per:(i + 1) * per])
                o.close()

            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=cores) as pool:
                list(pool.map(work, range(cores)))
            t_all += time.perf_counter() - t0
            n_all += per * cores
        out["cpu_baseline"] = {"value": n_all / t_all, "unit": "plans/s", "cores": cores, "kind": "oracle", "extrapolated": False,
                               "per_core_value": n_all / t_all / cores, "host_cores_available": os.cpu_count(),
                               "sample": "oracle cost of the first %d entries of every list, %d independent single-threaded workers (%.1f s)"
                                         % (per * cores, cores, t_all)}
    g.close()
    return out


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


# ---------------------------------------------------------------------------------------------------------
# exhaustive search over whole plan spaces (configs 1, 2, 3, 5)
# ---------------------------------------------------------------------------------------------------------
SEARCH_WORKLOADS = {
    "config1": ("config1: L=32 PP=4 DP=2 M=8, 1 failed node", lambda synth: [synth.config1()]),
    "config2": ("config2: L=48 PP=8 DP=4 M=16, 1 failed node", lambda synth: [synth.config2()]),
    "config3": ("config3: L=40 PP=4 DP=8 M=32, 2 failed nodes, Q16 speed factors, reroute cap 16", lambda synth: [synth.config3()]),
    "config5": ("config5: L=40 PP=8 DP=4 M=16, all 32 single and 496 double node failures",
                lambda synth: [synth.config5(fs) for fs in synth.config5_failure_sets()]),
}


def bench_search(args, B, synth, name):
    import numpy as np
    import torch
    label, make = SEARCH_WORKLOADS[name]
    scenarios = [dict(sc, transfer_assign=args.transfer_assign) for sc in make(synth)]
    if args.transfer_assign:
        label += ", least-transfer assignment"
    t0 = time.perf_counter()
    handles = [B.Scenario(sc) for sc in scenarios]
    load_ms = (time.perf_counter() - t0) * 1e3
    note("%s: %d scenario(s) loaded in %.1f ms" % (name, len(handles), load_ms))
    stream = torch.cuda.Stream()
    many = len(handles) > 1

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

    def one_step():
        """one search of every scenario: a single call for one scenario, one batched call for many"""
        if many:
            return B.search_best_batch(handles, 7, stream=stream)
        return [handles[0].search_best(7, stream=stream)]

    if args.copy_calibration:
        copy_calibration()
    with torch.cuda.stream(stream):
        for i in range(args.warmup):
            one_step()
        note("%s: warm-up done" % name)
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            plans = one_step()
        stream.synchronize()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        # Per-strategy kernel times (HIP events recorded by the library on this stream): the same searches again, one
        # handle at a time with event timing switched on, outside the timed region: each pair of events then brackets
        # one kernel running alone (in a batched step the kernels of different handles overlap on the library's side
        # streams).
        for g in handles:
            g.set_timing(True)
        fam_ms = np.zeros(3)
        serial_t0 = time.perf_counter()
        for _ in range(args.steps):
            for g in handles:
                g.search_best(7, stream=stream)
                fam_ms += np.array(g.get_timing()["family_ms"])
        serial_ms = (time.perf_counter() - serial_t0) * 1e3 / args.steps
        for g in handles:
            g.set_timing(False)
    ms_per_step = wall * 1e3 / args.steps
    fam_ms /= args.steps
    note("%s: timed %d steps: %.3f ms per step, kernel ms per strategy %s" % (name, args.steps, ms_per_step, fam_ms))
    cache_file = args.plan_cache
    if cache_file is None and many and os.path.isdir(os.path.join(ROOT, "gpurun_out")):
        cache_file = os.path.join(ROOT, "gpurun_out", "plan_cache_%s.jsonl" % name)
    if cache_file:
        with open(cache_file, "w") as fh:
            for sc_i, (rc_i, best_i) in zip(scenarios, plans):
                fh.write(json.dumps({"failed_nodes": sc_i["failed_nodes"], "rc": rc_i, "index": best_i["index"], "cost": best_i["cost"],
                                     "strategy": best_i["strategy"], "cuts": best_i["cuts"],
                                     "reroute": best_i["reroute"] if best_i["strategy"] == 2 else None}) + "\n")
        note("best plan of %d scenario(s) written to %s" % (len(plans), cache_file))

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
            # recurrence cells that run: the partitions that pass the memory filter, every pipeline class
            cells += tm["feasible"][f["strategy"]] * sum(2 * n * m for n, m in f["classes"])
    n_plans = float(evaluations.sum())

    # the per-call loop (one wait per scenario) beside the batched call
    per_call_ms = None
    if many and args.ttb_runs:
        with torch.cuda.stream(stream):
            t0 = time.perf_counter()
            for g in handles:
                g.search_best(7, stream=stream)
            per_call_ms = (time.perf_counter() - t0) * 1e3

    # time-to-best-plan: load + search on a fresh handle, median over --ttb-runs (first scenario)
    ttb = []
    for _ in range(args.ttb_runs):
        t0 = time.perf_counter()
        g2 = B.Scenario(scenarios[0])
        g2.search_best(7, stream=stream)
        ttb.append((time.perf_counter() - t0) * 1e3)
        g2.close()
    ttb_ms = float(np.median(ttb)) if ttb else None
    note("%s: time to best plan (load + search): %s ms" % (name, ttb_ms))

    # many scenarios: the host side of a call (launches, one synchronisation) hides behind other threads' kernels
    threaded_exhaustive = None
    if args.ttb_runs and many and args.threads:
        ms_t, same_t = threaded_sweep(B, handles, plans, reps=2)
        threaded_exhaustive = {"search_ms_all_scenarios_4_threads": ms_t, "same_plans": bool(same_t)}
        note("%s: exhaustive search from four host threads: %s" % (name, threaded_exhaustive))

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
            swept = [b for _, b in one_step()]
            search_b.append((time.perf_counter() - t0) * 1e3)
            same = same and all(a["index"] == b[1]["index"] and a["cost"] == b[1]["cost"] for a, b in zip(swept, plans))
        ev = np.zeros(3)
        for g in handles:
            ev += np.array(g.get_timing()["evaluated"], dtype=float)
        threaded_ms = None
        if many and args.threads:
            threaded_ms, same_t = threaded_sweep(B, handles, plans)
            same = same and same_t
        for g in handles:
            g.set_bounded_search(False)
        bounded = {"time_to_best_plan_ms": float(np.median(ttb_b)), "search_ms_all_scenarios": float(np.median(search_b)),
                   "search_ms_all_scenarios_4_threads": threaded_ms,
                   "partitions_evaluated_in_full": [float(x) for x in ev], "same_plans_as_exhaustive": bool(same)}
        note("%s: bounded search: %s" % (name, bounded))

    # roofline of the dominant kernel
    dom = int(np.argmax(fam_ms))
    achieved = ops[dom] / (fam_ms[dom] * 1e-3) / 1e12
    fam0 = [f for f in work[0] if f["strategy"] == dom]
    _, ops_light, ops_heavy = algorithmic_ops(fam0[0], 0) if fam0 else (0, 0, 0)
    probes = {pname: B.valu_probe(kind, 3000, stream=stream) / 1e12
              for kind, pname in ((0, "v_add_u32"), (1, "v_max_i32"), (2, "max_add_cell_chain"))}
    note("%s: measured VALU rates (T lane-ops/s): %s" % (name, probes))
    sc = scenarios[0]
    best = plans[0][1]
    shared = None
    if dom == 2 and fam0 and sum(fam0[0]["R"]) > 4096 and all(p >= 3 for p in fam0[0]["peers"]):
        # large reroute spaces are swept group by group (shared leading entries): the same figure with the operations
        # of that formulation in place of `peers` operations per reroute vector
        per_part = [shared_prefix_ops(p, t, sc0_cap) for p, t, sc0_cap in
                    zip(fam0[0]["peers"], fam0[0]["orphans"], [scenarios[0].get("reroute_cap", 0)] * len(fam0[0]["peers"]))]
        if all(x is not None for x in per_part):
            base_ops = algorithmic_ops(dict(fam0[0], R=[0] * len(fam0[0]["R"])), feasible[dom] / len(handles))[0]
            shared = (base_ops + feasible[dom] / len(handles) * sum(per_part)) * len(handles)
    roofline = {"bound": "alu", "kernel": "search, strategy %d" % dom, "achieved": achieved,
                "peak": ALU_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / ALU_PEAK_TOPS,
                "frac_is": "algorithmic int32 lane operations per second (the method's max/add/compare count, whatever the kernel "
                           "executes) over the nominal VALU peak of 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz; this is the figure "
                           "the 50 % target is read against",
                "measured_valu_rates_tops": probes,
                "algorithmic_ops_over_measured_naive_cell_rate": achieved / probes["max_add_cell_chain"],
                "algorithmic_ops_over_measured_naive_cell_rate_is": "the same numerator over the measured rate of a plain dependent "
                    "v_max_i32 + v_add_u32 chain; above 1 because the kernel executes fewer instructions than the algorithmic count "
                    "(one v_max serves a forward and a backward cell, the forward add folds into the frame, v_max3/v_min3 fold two operations)",
                "traffic": CONFIG2_TRAFFIC_BYTES[dom] if name == "config2" and not args.transfer_assign else None,
                "kernel_ms": float(fam_ms[dom]), "algorithmic_ops_per_launch": float(ops[dom] / len(handles)),
                "feasible_partitions": float(feasible[dom]),
                "algorithmic_ops_per_feasible_partition": ops_light + ops_heavy,
                "algorithmic_ops_per_infeasible_partition": ops_light}
    if shared is not None:
        a2 = shared / (fam_ms[dom] * 1e-3) / 1e12
        roofline["achieved_shared_prefix_accounting"] = a2
        roofline["frac_shared_prefix_accounting"] = a2 / ALU_PEAK_TOPS
        roofline["frac_shared_prefix_accounting_is"] = (
            "`frac` charges every reroute vector its `peers` operations (the accounting of all workloads); this kernel takes the "
            "largest product of the leading entries once per group of vectors and the best pair of the last two entries from a "
            "table, so it needs far fewer: with the operations of that formulation as the numerator the fraction is this one")
    if name == "config2" and not args.transfer_assign:
        per_part = CONFIG2_EXECUTED_LANE_INSTR_PER_PARTITION[dom]
        executed = per_part * fam0[0]["n_part"] / (fam_ms[dom] * 1e-3) / 1e12
        roofline["executed_lane_instr_per_partition"] = per_part
        roofline["executed_valu_rate_tops"] = executed
        roofline["executed_valu_rate_over_measured_v_max_rate"] = executed / probes["v_max_i32"]
        roofline["executed_valu_rate_is"] = ("SQ_INSTS_VALU x 64 / partitions of the committed rocprofv3 profile x partitions / kernel time "
                                             "of this run, against the measured issue rate of v_max_i32 (the slower of the two "
                                             "instruction classes the kernel mixes)")
    out = {
        "metric": METRIC,
        "value": n_plans / (ms_per_step * 1e-3),
        "unit": "plans/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int32", "data": "synthetic",
        "config": {"workload": label + ", exhaustive search over all strategies" + (", one batched call for all scenarios" if many else ""),
                   "scenarios": len(handles), "plans_scored_per_step": n_plans, "plan_indices": plan_indices,
                   "partitions": n_part_total, "failed_nodes": sc["failed_nodes"] if not many else "all",
                   "families": [{k: f[k] for k in ("strategy", "stages", "n_part", "n_reroute")} for f in work[0]]},
        "time_to_best_plan_ms": ttb_ms, "load_ms": load_ms,
        "load_ms_is": "first handle(s) of the process: includes HIP initialisation and loading the code object; "
                      "time_to_best_plan_ms is the warm load + search",
        "time_to_best_plan_bounded_ms": bounded["time_to_best_plan_ms"] if bounded else None,
        "bounded_search": bounded,
        "exhaustive_search_4_threads": threaded_exhaustive,
        "per_call_loop_ms": per_call_ms,
        "plan_cache_file": os.path.relpath(cache_file, ROOT) if cache_file else None,
        "kernels_one_after_the_other_ms": float(fam_ms.sum()),
        "kernels_one_after_the_other_is": "sum of the strategy kernels' own durations (each measured running alone); in a batched step "
                                          "the kernels of different scenarios overlap on the library's side streams, so ms_per_step "
                                          "can be below this sum",
        "per_call_loop_with_timing_ms": serial_ms,
        "partition_evals_per_s": n_part_total / (ms_per_step * 1e-3),
        "recurrence_cells_per_s": cells / (ms_per_step * 1e-3),
        "kernel_ms_per_strategy": [float(x) for x in fam_ms],
        "best": {"index": best["index"], "cost": best["cost"], "strategy": best["strategy"], "cuts": best["cuts"]},
        "roofline": roofline,
        "feasible_partitions_per_strategy": [float(x) for x in feasible],
        "filter_compaction": {"mode": args.filter_compaction, "sampled_fit_share": fit_share},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_record(scenarios[0], args.cpu_seconds, name + (" (first scenario)" if many else ""))
    for g in handles:
        g.close()
    return out


def summary(rec):
    """what the `workloads` block keeps of a workload's record"""
    keep = ("value", "unit", "steps", "ms_per_step", "time_to_best_plan_ms", "time_to_best_plan_bounded_ms", "partition_evals_per_s",
            "recurrence_cells_per_s", "kernel_ms_per_strategy", "ms_per_strategy", "search_kernels_ms", "per_call_loop_ms",
            "plan_cache_file", "kernels_one_after_the_other_ms", "replan_table_1_to_3", "cpu_baseline")
    out = {k: rec[k] for k in keep if k in rec and rec[k] is not None}
    out["workload"] = rec["config"]["workload"]
    r = rec["roofline"]
    out["roofline"] = {k: r[k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac", "kernel_ms", "achieved_shared_prefix_accounting",
                                         "frac_shared_prefix_accounting", "frac_shared_prefix_accounting_is") if k in r}
    if rec.get("bounded_search"):
        b = rec["bounded_search"]
        out["bounded_search"] = {k: b[k] for k in ("search_ms_all_scenarios", "bounded_ms_per_step", "time_to_best_plan_ms",
                                                   "same_plans_as_exhaustive", "same_winners", "same_plan_as_exhaustive") if k in b}
    return out


def run_workload(name, args, B, synth):
    if name == "replan32":
        return bench_replan(args, B, synth)
    if name == "score2":
        return bench_score(args, B, synth)
    if name == "config4":
        return bench_lists(args, B, synth)
    return bench_search(args, B, synth, name)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--ttb-runs", type=int, default=10)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2", "config3", "config4", "config5", "replan32", "score2"],
                    help="config2 (the 32-card shape) is the benchmark; the others are reported in its `workloads` block and can be "
                         "run alone for profiling; replan32 times chm_replan (search over DP/PP degrees) for the 31 nodes that "
                         "survive in config2")
    ap.add_argument("--no-workloads", action="store_true", help="config2 only, without the `workloads` block")
    ap.add_argument("--threads", action="store_true", help="many scenarios: also time four host threads with a stream each")
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

    import torch
    from paper_2508_21613_amd import binding as B
    from paper_2508_21613_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    out = run_workload(args.workload, args, B, synth)
    if args.workload == "config2" and not args.no_workloads:
        # the other configurations at a few steps each, with a short oracle sample
        sub = argparse.Namespace(**vars(args))
        sub.steps, sub.warmup, sub.ttb_runs, sub.cpu_seconds, sub.copy_calibration, sub.plan_cache = 3, 1, 3, 3.0, False, None
        block = {}
        for name in ("config1", "config3", "config4", "config5", "score2", "replan32"):
            t0 = time.perf_counter()
            block[name] = summary(run_workload(name, sub, B, synth))
            note("workload %s done in %.1f s" % (name, time.perf_counter() - t0))
        out["workloads"] = block
    print(json.dumps(out))


if __name__ == "__main__":
    main()
