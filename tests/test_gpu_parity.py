"""Parity of the HIP library (through its C-ABI) with the CPU oracle, bit for bit.

All costs are integers, so every comparison is exact: every plan cost of the small
scenarios, seeded windows of the five benchmark configurations, and the (index, cost,
cuts, reroute vectors) of every argmin.
"""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2508_21613_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2508_21613_amd import binding
    binding.lib()
    return binding


def gpu_scores(B, g, first, count):
    import torch
    out = g.score_plans(first, count)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def same_plan(a, b):
    keys = ("index", "cost", "strategy", "stages", "cuts", "n_affected", "affected_stage", "reroute", "t_step_us", "t_trans_us")
    return all(a[k] == b[k] for k in keys)


SMALL = [synth.small_random(1000 + i) for i in range(24)] + [
    synth.small_random(2000, L=7, PP=3, DP=3, M=4, n_failed=2, hetero=True, cap=3),
    synth.small_random(2001, L=6, PP=3, DP=4, M=3, n_failed=2, hetero=True, cap=0),
    synth.small_random(2002, L=8, PP=4, DP=2, M=5, n_failed=1, hetero=False),
    synth.small_random(2003, L=6, PP=2, DP=3, M=6, n_failed=3, hetero=True, cap=7),
    synth.small_random(2004, L=12, PP=5, DP=3, M=2, n_failed=2, hetero=True),       # M < S-1
    synth.small_random(2005, L=10, PP=9, DP=2, M=3, n_failed=1, hetero=False),      # nearly one layer per stage
    synth.small_random(2006, L=9, PP=9, DP=2, M=4, n_failed=1, hetero=True),        # exactly one partition
    synth.small_random(2007, L=6, PP=1, DP=3, M=5, n_failed=1, hetero=True),        # single-stage pipelines
    synth.small_random(2008, L=14, PP=6, DP=4, M=7, n_failed=4, hetero=True, cap=9),
    synth.small_random(2009, L=20, PP=12, DP=2, M=13, n_failed=2, hetero=True),     # > 8 stages
    synth.small_random(2010, L=22, PP=18, DP=2, M=5, n_failed=1, hetero=False),     # > 16 stages
    synth.small_random(2011, L=16, PP=10, DP=3, M=12, n_failed=2, hetero=True),
    synth.small_random(2012, L=18, PP=14, DP=2, M=20, n_failed=1, hetero=True),
    synth.small_random(2013, L=15, PP=11, DP=2, M=4, n_failed=2, hetero=False),     # M < S-1 on the unrolled path
]


def _two_lost_in_one_pipeline():
    # pipeline 0 loses stages 1 and 4 (not ring-adjacent): the redundant strategy runs a chain of S-2 nodes
    fwd, bwd, mem = synth.layer_tables(4242, 13)
    return synth.scenario(13, 6, 3, 7, fwd, bwd, mem, [1, 4], 120, int(mem.sum() * 2.2 / 6),
                          speed=synth.speed_factors(4242, 3, 6))


SMALL.append(_two_lost_in_one_pipeline())
SMALL.append(dict(_two_lost_in_one_pipeline(), failed_nodes=[0, 3, 8], M=3))


SMALL_ACT = [synth.with_activations(sc, 3000 + i) for i, sc in enumerate(SMALL)]
# least-transfer assignment of survivors to new stages, alternately without and with activation memory
SMALL_KM = [dict(SMALL_ACT[i] if i % 2 else sc, transfer_assign=1) for i, sc in enumerate(SMALL)]
# rounds of gradient communication in the step time, on top of the three variants above in turn
SMALL_AR = [dict((SMALL, SMALL_ACT, SMALL_KM)[i % 3][i], allreduce_us=250 + 35 * i) for i in range(len(SMALL))]
ALL_SMALL = SMALL + SMALL_ACT + SMALL_KM + SMALL_AR


@pytest.mark.parametrize("i", range(len(ALL_SMALL)))
def test_small_scenarios_every_cost_and_argmin(B, i):
    sc = ALL_SMALL[i]
    print("small scenario", i, {k: sc.get(k) for k in ("L", "PP", "DP", "M", "failed_nodes", "reroute_cap", "transfer_assign", "allreduce_us")}, flush=True)
    o = O.Scenario(sc)
    g = B.Scenario(sc)
    assert g.families == o.families and g.n_plans == o.n_plans
    n = min(o.n_plans, 60000)
    want = o.score(0, n)
    got = gpu_scores(B, g, 0, n)
    assert (got == want).all(), np.flatnonzero(got != want)[:10]
    for mask in [7] + [1 << f["strategy"] for f in o.families]:
        rc_o, best_o = o.search(mask)
        rc_g, best_g = g.search_best(mask)
        assert rc_g == rc_o, (mask, rc_g, rc_o)
        assert same_plan(best_g, best_o), (mask, best_g, best_o)
    # bounded search: the same plans, ties included; mode 2 takes the seeds and the enumeration of candidates
    # at these small sizes too
    g.set_timing(True)
    for mode in (1, 2):
        g.set_bounded_search(mode)
        for mask in [7] + [1 << f["strategy"] for f in o.families]:
            rc_o, best_o = o.search(mask)
            rc_g, best_g = g.search_best(mask)
            assert rc_g == rc_o and same_plan(best_g, best_o), ("bounded", mode, mask, best_g, best_o)
            t = g.get_timing()
            assert all(e <= f for e, f in zip(t["evaluated"], t["feasible"]))
        for f in o.families:
            lo, n = f["n_part"] // 3, max(1, f["n_part"] // 2)
            rc_o, best_o, _ = o.search_range(f["strategy"], lo, n)
            rc_g, best_g = g.search_range(f["strategy"], lo, n)
            assert rc_g == rc_o and same_plan(best_g, best_o), ("bounded range", mode, f["strategy"], best_g, best_o)
    g.set_bounded_search(0)
    for idx in range(0, o.n_plans, max(1, o.n_plans // 25)):
        d_o, d_g = o.decode(idx), g.decode_plan(idx)
        d_o.update(cost=0, t_step_us=0, t_trans_us=0)      # the library's decoding is structural only
        assert same_plan(d_g, d_o)


def _uniform_layers(sc, cap):
    """the same scenario with identical layers and free weight transfer (many plans of equal cost) and the given memory cap"""
    L = sc["L"]
    return dict(sc, fwd_us=[1000] * L, bwd_us=[2000] * L, mem_mib=[500] * L, mem_cap_mib=cap, act_mib=None, xfer_us_per_mib=0)


COMPACTION = [
    ("config2", lambda: synth.config2()),
    ("config2_tight", lambda: dict(synth.config2(), mem_cap_mib=6600)),           # few partitions fit
    ("config2_none_fit", lambda: dict(synth.config2(), mem_cap_mib=2000)),
    ("config2_act_allreduce", lambda: dict(synth.with_activations(synth.config2(), 31), allreduce_us=900)),
    ("config5_double_assign", lambda: dict(synth.config5([3, 17]), transfer_assign=1)),
    ("config3", lambda: synth.config3()),
    ("config3_cap12", lambda: dict(synth.config3(), reroute_cap=12)),
    ("config3_uncapped_m8", lambda: dict(synth.config3(), reroute_cap=0, M=8)),
    ("config4", lambda: synth.config4(mem_cap_mib=synth.CONFIG4_CAP_30PCT)),
    ("config1_ties", lambda: _uniform_layers(synth.config1(), 9000)),
    ("config2_ties", lambda: _uniform_layers(synth.config2(), 8000)),
    ("small_6_stages", lambda: synth.small_random(4242, L=20, PP=6, DP=3, M=7, n_failed=1, hetero=True)),
]


@pytest.mark.parametrize("name", [c[0] for c in COMPACTION])
def test_filter_compaction_modes_agree_with_the_oracle(B, name):
    """range search of strategies 0 and 1 with the partitions that fit compacted per wavefront (mode 1) and
    without (mode 0): same winner as the oracle on seeded windows (lowest index among equal costs), same count
    of partitions that fit, and the same winner over the whole space in both modes."""
    sc = dict(COMPACTION)[name]()
    o, g = O.Scenario(sc), B.Scenario(sc)
    g.set_timing(True)
    rng = np.random.default_rng(11)
    share = g.set_filter_compaction(-1)
    print("compaction", name, "sampled share of partitions that fit", share, flush=True)
    for f in o.families:
        if f["strategy"] == 2:
            continue
        width = min(f["n_part"], 30000)
        firsts = {0, f["n_part"] - width} | {int(rng.integers(0, f["n_part"] - width + 1)) for _ in range(3)}
        for first in sorted(firsts):
            rc_o, best_o, _ = o.search_range(f["strategy"], first, width)
            fit = None
            for mode in (1, 0):
                g.set_filter_compaction(mode)
                rc_g, best_g = g.search_range(f["strategy"], first, width)
                assert rc_g == rc_o, (name, f["strategy"], first, mode, rc_g, rc_o)
                assert same_plan(best_g, best_o), (name, f["strategy"], first, mode, best_g, best_o)
                n_fit = g.get_timing()["feasible"][f["strategy"]]
                assert fit is None or n_fit == fit
                fit = n_fit
        if f["n_part"] > 2 * 10 ** 8:          # config 4: the whole space is out of reach, the windows stand for it
            g.set_filter_compaction(1)
            with pytest.raises(B.ChmError) as err:
                g.search_best(1 << f["strategy"])
            assert err.value.code == B.ERR_OVERFLOW
            continue
        whole = []
        for mode in (1, 0, -1):
            g.set_filter_compaction(mode)
            rc, best = g.search_best(1 << f["strategy"])
            whole.append((rc, best, g.get_timing()["feasible"][f["strategy"]]))
        assert whole[0][0] == whole[1][0] == whole[2][0]
        assert same_plan(whole[0][1], whole[1][1]) and same_plan(whole[0][1], whole[2][1])
        assert whole[0][2] == whole[1][2] == whole[2][2]
        if whole[0][0] == 0:
            best = whole[0][1]
            assert o.decode(best["index"])["cost"] == best["cost"]
            # the window around the winner: the oracle finds the same plan there, in both modes
            part = best["index"] - f["offset"]
            first = max(0, min(part - width // 2, f["n_part"] - width))
            rc_o, best_o, _ = o.search_range(f["strategy"], first, width)
            assert rc_o == 0 and same_plan(best, best_o), (name, f["strategy"], best, best_o)
            for mode in (1, 0):
                g.set_filter_compaction(mode)
                rc_g, best_g = g.search_range(f["strategy"], first, width)
                assert rc_g == 0 and same_plan(best_g, best_o)


@pytest.mark.parametrize("name", [c[0] for c in COMPACTION])
def test_bounded_search_returns_the_exhaustive_winner(B, name):
    """chm_set_bounded_search skips partitions whose lower bound of the cost lies above the best cost found so
    far: same winner as the oracle on seeded windows and as the exhaustive search over the whole space, for every
    strategy and for all of them together; fewer partitions evaluated than fit, never more."""
    sc = dict(COMPACTION)[name]()
    o, g = O.Scenario(sc), B.Scenario(sc)
    g.set_timing(True)
    rng = np.random.default_rng(12)
    reachable = all(f["n_part"] <= 2 * 10 ** 8 for f in o.families)
    for f in o.families:
        width = min(f["n_part"], 30000 if f["n_reroute"] < 1000 else 300)
        firsts = {0, f["n_part"] - width} | {int(rng.integers(0, f["n_part"] - width + 1)) for _ in range(3)}
        for first in sorted(firsts):
            rc_o, best_o, _ = o.search_range(f["strategy"], first, width)
            g.set_bounded_search(True)
            rc_g, best_g = g.search_range(f["strategy"], first, width)
            t = g.get_timing()
            assert rc_g == rc_o and same_plan(best_g, best_o), (name, f["strategy"], first, best_g, best_o)
            assert t["evaluated"][f["strategy"]] <= t["feasible"][f["strategy"]]
            assert rc_g != 0 or t["evaluated"][f["strategy"]] >= 1
    if not reachable:
        return
    masks = [7] + [1 << f["strategy"] for f in o.families]
    for mask in masks:
        g.set_bounded_search(False)
        rc_e, best_e = g.search_best(mask)
        t_e = g.get_timing()
        g.set_bounded_search(True)
        rc_b, best_b = g.search_best(mask)
        t_b = g.get_timing()
        assert rc_b == rc_e and same_plan(best_b, best_e), (name, mask, best_b, best_e)
        assert all(b <= e for b, e in zip(t_b["feasible"], t_e["feasible"])) and t_e["evaluated"] == t_e["feasible"]
        assert all(b <= e for b, e in zip(t_b["evaluated"], t_e["evaluated"]))
        print("bounded", name, "mask", mask, "fit", t_b["feasible"], "evaluated", t_b["evaluated"],
              "ms", [round(x, 3) for x in t_e["family_ms"]], "->", [round(x, 3) for x in t_b["family_ms"]], flush=True)


@pytest.mark.parametrize("seed", range(7000, 7030))
def test_bounded_search_on_seeded_mid_size_scenarios(B, seed):
    """random shapes of 10^3..10^5 partitions per strategy (heterogeneous speeds, one or two failures, in turn with
    activation memory, least-transfer assignment and communication rounds): the bounded search, with and
    without its size thresholds, returns the oracle's exhaustive argmin"""
    PP = 4 + seed % 3
    sc = synth.small_random(seed, L=PP + 10 + seed % 8, PP=PP, DP=2 + seed % 3, M=3 + seed % 14)
    if seed % 3 == 0:
        sc = synth.with_activations(sc, seed)
    if seed % 4 == 0:
        sc = dict(sc, transfer_assign=1)
    if seed % 5 == 0:
        sc = dict(sc, allreduce_us=300 + seed % 700)
    print("mid-size scenario", seed, {k: sc.get(k) for k in ("L", "PP", "DP", "M", "failed_nodes")}, flush=True)
    o, g = O.Scenario(sc), B.Scenario(sc)
    for mask in [7] + [1 << f["strategy"] for f in o.families]:
        rc_o, best_o = o.search(mask)
        for mode in (1, 2):
            g.set_bounded_search(mode)
            rc_g, best_g = g.search_best(mask)
            assert rc_g == rc_o and same_plan(best_g, best_o), (seed, mask, mode, best_g, best_o)


def test_bounded_search_over_the_whole_space_of_config4(B):
    """L=96 on 16 (15) stages: 10^17 partitions per strategy, out of reach of the exhaustive search
    (CHM_ERR_OVERFLOW).  The bounded search enumerates only the partitions whose lower bound of the cost does not
    exceed the best seed's cost.  The oracle cannot enumerate the space either, so: the winner's cost is
    recomputed by the oracle from its cuts, the oracle's argmin over the window of ranks around it is the same
    plan, no plan of seeded windows elsewhere is better, and no single cut can be moved by one layer to a
    better plan."""
    sc = synth.config4(mem_cap_mib=synth.CONFIG4_CAP_30PCT)
    o, g = O.Scenario(sc), B.Scenario(sc)
    g.set_bounded_search(True)
    g.set_timing(True)
    rng = np.random.default_rng(21)
    reached = 0
    for f in o.families:
        try:
            rc, best = g.search_best(1 << f["strategy"])
        except B.ChmError as err:
            assert err.code == B.ERR_OVERFLOW
            print("config4 whole space, strategy", f["strategy"], "too many candidates", flush=True)
            continue
        t = g.get_timing()
        print("config4 whole space, strategy", f["strategy"], "rc", rc, "cost", best["cost"], "cuts", best["cuts"],
              "candidates that fit", t["feasible"][f["strategy"]], flush=True)
        if rc != 0:
            continue
        reached += 1
        rr = best["reroute"] if best["strategy"] == 2 else None
        assert o.plan_cost(best["strategy"], best["cuts"], rr) == best["cost"]
        assert o.decode(best["index"])["cost"] == best["cost"]
        part = (best["index"] - f["offset"]) // f["n_reroute"]
        width = 20000 if f["n_reroute"] == 1 else 300
        first = max(0, min(part - width // 2, f["n_part"] - width))
        rc_o, best_o, _ = o.search_range(f["strategy"], first, width)
        assert rc_o == 0 and same_plan(best, best_o)
        for _ in range(4):
            first = int(rng.integers(0, f["n_part"] - width))
            rc_o, w, _ = o.search_range(f["strategy"], first, width)
            assert rc_o != 0 or (w["cost"], w["index"]) >= (best["cost"], best["index"])
        cuts = best["cuts"]
        for i in range(len(cuts)):
            for delta in (-1, 1):
                c2 = list(cuts)
                c2[i] += delta
                if c2 != sorted(set(c2)) or c2[0] < 1 or c2[-1] > sc["L"] - 1:
                    continue
                rc_o, w, _ = o.search_range(f["strategy"], int(O.partition_rank(c2)), 1)
                assert rc_o != 0 or (w["cost"], w["index"]) >= (best["cost"], best["index"])
    assert reached >= 1


def test_equal_costs_in_an_explicit_list_go_to_the_lowest_position(B):
    """a list in which the best partition occurs many times at seeded positions: the reported position is
    the first of them, whatever order the compacted entries are evaluated in"""
    import torch
    for sc in (synth.config4(mem_cap_mib=synth.CONFIG4_CAP_30PCT), synth.config2()):
        o, g = O.Scenario(sc), B.Scenario(sc)
        for f in o.families:
            if f["n_reroute"] != 1:
                continue
            k = f["stages"] - 1
            n = 40000
            cuts = synth.random_partitions(91, 3 + f["strategy"], n, sc["L"], k)
            want = o.score_ranks(f["strategy"], O.partition_rank_batch(cuts))
            if (want == O.INF).all():
                continue
            winner = cuts[int(np.argmin(want))].copy()
            where = np.random.default_rng(5 + f["strategy"]).choice(np.arange(2000, n), size=300, replace=False)
            cuts[where] = winner
            want[where] = want.min()
            costs = torch.empty(n, dtype=torch.int64, device="cuda")
            rc, best, pos = g.search_cuts(f["strategy"], torch.from_numpy(cuts).cuda(), costs=costs)
            assert rc == 0 and (costs.cpu().numpy() == want).all()
            assert pos == int(np.argmin(want)), (f["strategy"], pos, int(np.argmin(want)))
            assert best["cuts"] == [int(x) for x in winner] and best["cost"] == int(want.min())
            g.set_bounded_search(1)
            rc_b, best_b, pos_b = g.search_cuts(f["strategy"], torch.from_numpy(cuts).cuda())
            g.set_bounded_search(0)
            assert rc_b == 0 and pos_b == pos and same_plan(best_b, best)


def test_config1_all_9455_plans(B):
    sc = synth.config1()
    o, g = O.Scenario(sc), B.Scenario(sc)
    assert g.n_plans == 9455
    want = o.score(0, 9455)
    got = gpu_scores(B, g, 0, 9455)
    assert (got == want).all()
    assert (want == O.INF).sum() > 0 and (got == B.INFEASIBLE).sum() == (want == O.INF).sum()
    rc_o, best_o = o.search(7)
    rc_g, best_g = g.search_best(7)
    assert rc_o == rc_g == 0 and same_plan(best_g, best_o)
    # ragged sub-ranges, including ones that straddle family boundaries and an empty one
    for first, count in [(0, 1), (4494, 3), (4900, 130), (9454, 1), (17, 0), (3000, 777)]:
        assert (gpu_scores(B, g, first, count) == want[first:first + count]).all()


def windows(o, rng, n_windows, width):
    """seeded windows of the plan space, plus the ends and the family boundaries"""
    out = [(0, width), (o.n_plans - width, width)]
    for f in o.families[1:]:
        out.append((f["offset"] - width // 2, width))
    for _ in range(n_windows):
        out.append((int(rng.integers(0, o.n_plans - width)), width))
    return out


@pytest.mark.parametrize("name", ["config2", "config3", "config5_single", "config5_double", "config2_act", "config3_act",
                                  "config2_assign", "config3_assign", "config5_double_assign",
                                  "config2_allreduce", "config3_allreduce", "config5_double_allreduce"])
def test_seeded_windows_of_the_large_configs(B, name):
    sc = {"config2": synth.config2, "config3": synth.config3,
          "config2_assign": lambda: dict(synth.config2(), transfer_assign=1),
          "config3_assign": lambda: dict(synth.with_activations(synth.config3(), 79), transfer_assign=1),
          "config5_double_assign": lambda: dict(synth.config5([3, 30]), transfer_assign=1),
          "config2_allreduce": lambda: dict(synth.config2(), allreduce_us=1500),
          "config3_allreduce": lambda: dict(synth.with_activations(synth.config3(), 80), allreduce_us=900, transfer_assign=1),
          "config5_double_allreduce": lambda: dict(synth.config5([6, 7]), allreduce_us=2500),

          "config2_act": lambda: synth.with_activations(synth.config2(), 77),
          "config3_act": lambda: synth.with_activations(synth.config3(), 78),
          "config5_single": lambda: synth.config5([13]),
          "config5_double": lambda: synth.config5([5, 26])}[name]()
    print(name, "failed", sc["failed_nodes"], flush=True)
    o, g = O.Scenario(sc), B.Scenario(sc)
    assert g.families == o.families and g.n_plans == o.n_plans
    rng = np.random.default_rng(42)
    width = 700 if o.n_plans > 1400 else o.n_plans // 2
    wins = windows(o, rng, 6, width)
    if name.endswith("_assign"):                    # the assignment only changes the re-partition strategy: look there
        f1 = o.family(1)
        wins += [(f1["offset"] + int(rng.integers(0, f1["n_part"] - width)), width) for _ in range(6)]
    for first, count in wins:
        want = o.score(first, count)
        got = gpu_scores(B, g, first, count)
        assert (got == want).all(), (first, np.flatnonzero(got != want)[:5])
    # argmin over sub-ranges of partitions, family by family
    for f in o.families:
        width = 40 if (f["strategy"] == 2 and f["n_reroute"] > 10 ** 6) else 3000
        width = min(width, f["n_part"])
        for first in (0, f["n_part"] - width, int(rng.integers(0, f["n_part"] - width + 1))):
            print(name, "search_range", f["strategy"], first, width, flush=True)
            rc_o, best_o, _ = o.search_range(f["strategy"], first, width)
            rc_g, best_g = g.search_range(f["strategy"], first, width)
            assert rc_g == rc_o and same_plan(best_g, best_o), (f, first, best_g, best_o)


@pytest.mark.parametrize("cap,assign,allreduce", [(6000, 0, 0), (synth.CONFIG4_CAP_30PCT, 0, 0), (synth.CONFIG4_CAP_30PCT, 1, 0),
                                                  (synth.CONFIG4_CAP_30PCT, 0, 1200)])
def test_config4_explicit_partitions(B, cap, assign, allreduce):
    import torch
    sc = dict(synth.config4(mem_cap_mib=cap), transfer_assign=assign, allreduce_us=allreduce)
    o, g = O.Scenario(sc), B.Scenario(sc)
    assert g.families == o.families
    n = 3000
    for strategy, k in ((0, 15), (1, 14), (2, 15)):
        cuts = synth.random_partitions(synth.BASE_SEED + 4, 20 + strategy, n, 96, k)
        ranks = np.array([O.partition_rank(c) for c in cuts], dtype=np.uint64)
        want = o.score_ranks(strategy, ranks)
        d_ranks = torch.from_numpy(ranks.view(np.int64)).cuda()
        got = g.score_ranks(strategy, d_ranks)
        torch.cuda.synchronize()
        got = got.cpu().numpy()
        assert (got == want).all(), np.flatnonzero(got != want)[:5]
        frac = (want == O.INF).mean()
        print("config4 strategy", strategy, "infeasible fraction", frac, flush=True)
    # a rank outside the family is reported as infeasible, not as an error
    bad = torch.tensor([0, 2 ** 62], dtype=torch.int64, device="cuda")
    got = g.score_ranks(1, bad).cpu().numpy()
    assert got[1] == B.INFEASIBLE and got[0] == o.score_ranks(1, [0])[0]


@pytest.mark.parametrize("assign,allreduce", [(0, 0), (1, 0), (0, 1500)])
def test_full_size_search_config2(B, assign, allreduce):
    """the 32-card shape, whole space, in the launch configuration the benchmark times:
    the winner is re-scored plan by plan by the oracle, is compared with the oracle's argmin
    over the windows around it, and must not be beaten by any plan of a seeded sample."""
    sc = dict(synth.config2(), transfer_assign=assign, allreduce_us=allreduce)
    o, g = O.Scenario(sc), B.Scenario(sc)
    rc, best = g.search_best(7)
    assert rc == 0
    print("config2 best", best["index"], best["cost"], best["strategy"], best["cuts"], flush=True)
    rr = best["reroute"] if best["strategy"] == 2 else None
    assert o.plan_cost(best["strategy"], best["cuts"], rr) == best["cost"]
    assert o.decode(best["index"])["cost"] == best["cost"]
    fam = o.family(best["strategy"])
    part = (best["index"] - fam["offset"]) // fam["n_reroute"]
    lo = max(0, part - 20000)
    rc_o, best_o, _ = o.search_range(best["strategy"], lo, min(40000, fam["n_part"] - lo))
    assert rc_o == 0 and same_plan(best, best_o)
    rng = np.random.default_rng(5)
    for f in o.families:
        rc_f, best_f = g.search_best(1 << f["strategy"])
        assert rc_f == 0 and best_f["cost"] >= best["cost"]
        assert o.decode(best_f["index"])["cost"] == best_f["cost"]
        for _ in range(4):
            first = int(rng.integers(0, f["n_part"] - 5000))
            rc_o, w, _ = o.search_range(f["strategy"], first, 5000)
            if rc_o == 0:
                assert (w["cost"], w["index"]) >= (best_f["cost"], best_f["index"])


def test_migration_scheme_of_the_re_partition_strategy(B):
    """chm_transfer_plan: the assignment must be one-to-one, fetch exactly what it reports, and that
    total must be the oracle's minimum over all assignments (transfer_assign = 1) or the stage-order
    total (0).  Several optimal assignments can exist, so only the total is compared."""
    rng = np.random.default_rng(21)
    cases = [dict(sc, transfer_assign=a) for a in (1, 0) for sc in (SMALL[3], SMALL[24], SMALL[30], SMALL[33], SMALL[38], SMALL[39])]
    cases += [dict(synth.config2(), transfer_assign=1), dict(synth.config5([3, 30]), transfer_assign=1),
              dict(synth.config4(mem_cap_mib=synth.CONFIG4_CAP_30PCT), transfer_assign=1)]
    checked = improved = 0
    for sc in cases:
        g, o = B.Scenario(sc), O.Scenario(sc)
        f = o.family(1)
        if f is None:
            continue
        S, L, n = sc["PP"], sc["L"], f["stages"]
        p0 = O.layout_p0(L, S)
        lost = sorted({x // S for x in sc["failed_nodes"]})
        print("migration scheme", {k: sc[k] for k in ("L", "PP", "DP", "failed_nodes", "transfer_assign")}, flush=True)
        ranks = [0, f["n_part"] - 1] + [int(rng.integers(0, f["n_part"])) for _ in range(12)]
        for d in lost:
            alive = [j for j in range(S) if d * S + j not in sc["failed_nodes"]]
            for r in ranks:
                node_stage, stage_of, mib = g.transfer_plan(r, d)
                assert node_stage == alive and sorted(stage_of) == list(range(n))
                b = [0] + O.partition_unrank(L, n - 1, r) + [L]
                fetch = [[O.missing_interval(sc["mem_mib"], b[j], b[j + 1], p0[h], p0[h + 1]) for j in range(n)] for h in alive]
                assert sum(fetch[i][stage_of[i]] for i in range(n)) == mib
                in_order = sum(fetch[j][j] for j in range(n))
                if sc["transfer_assign"]:
                    assert mib == O.min_assignment(fetch)[0] <= in_order
                    improved += mib < in_order
                else:
                    assert mib == in_order and stage_of == list(range(n))
                checked += 1
        intact = [d for d in range(sc["DP"]) if d not in lost]
        if intact:
            with pytest.raises(B.ChmError) as e:
                g.transfer_plan(0, intact[0])
            assert e.value.code == B.ERR_ARG
        with pytest.raises(B.ChmError) as e:
            g.transfer_plan(f["n_part"], lost[0])
        assert e.value.code == B.ERR_RANGE
    assert checked > 150 and improved > 0


REPLAN = [
    synth.replan_case(5, 10, 3, 3, [4], 12, (1, 4), (1, 6)),
    synth.replan_case(6, 9, 2, 4, [1], 16, (1, 4), (1, 8), act=True),
    synth.replan_case(7, 12, 4, 2, [3], 16, (2, 5), (1, 4)),
    synth.replan_case(8, 11, 3, 3, [0, 5], 9, (1, 5), (1, 7), horizon_us=20_000_000),
    synth.replan_case(9, 8, 2, 3, [2, 3, 4], 6, (1, 3), (1, 3), act=True),
    synth.replan_case(10, 13, 2, 5, [7], 10, (1, 3), (2, 6), dist="lognormal"),
    synth.replan_case(11, 10, 3, 2, [], 12, (1, 6), (1, 6)),
    synth.replan_case(12, 9, 3, 3, [8], 7, (2, 4), (1, 5), xfer_us_per_mib=5000, horizon_us=60_000_000),
    synth.replan_case(13, 12, 3, 4, [2, 6], 3, (1, 5), (1, 10)),
    synth.replan_case(14, 10, 2, 4, [0], 8, (1, 4), (1, 7), cap_scale=0.9),
    synth.replan_case(15, 14, 4, 4, [5, 10], 24, (2, 7), (1, 7), act=True),               # 14 nodes, up to 7 pipelines
    synth.replan_case(16, 16, 8, 4, [0, 9, 18, 27], 64, (5, 9), (2, 6)),                   # 28 nodes
    synth.replan_case(17, 12, 16, 4, list(range(0, 64, 7)), 96, (12, 16), (3, 5)),         # 54 nodes, 16 pipelines
    synth.replan_case(18, 6, 2, 2, [0, 1, 2, 3], 4, (1, 2), (1, 2)),                       # nothing survived
    synth.replan_tie(),                                                                     # two candidates tie exactly
    synth.replan_case(19, 12, 3, 4, [5], 700, (2, 5), (2, 6), cap_scale=4.5),       # 11 nodes, 700 micro-batches: with 2 pipelines one of them would run more than 256
    synth.replan_case(20, 11, 3, 4, [5], 20, (2, 5), (1, 6)),       # 11 nodes: no pipeline count in range divides them
    synth.replan_case(21, 12, 3, 4, [5], 3000, (2, 5), (2, 6), cap_scale=4.5),   # every layout overloads a pipeline: no candidate
]


@pytest.mark.parametrize("i", range(len(REPLAN)))
def test_replan_over_dp_pp_degrees(B, i):
    """chm_replan against the oracle's Algorithm 1: every field of the chosen plan is an integer that
    both sides fix uniquely (first minimum in rank order per pipeline, smaller dp on ties)"""
    rp = REPLAN[i]
    print("replan", i, {k: rp[k] for k in ("L", "old_dp", "old_pp", "failed_nodes", "dp_min", "dp_max", "pp_min", "pp_max", "micro_batches")}, flush=True)
    want = O.replan(rp)
    got = B.replan(rp)
    assert got == want, (got, want)
    for H in (3 * 10 ** 7, 10 ** 11):
        assert B.replan(dict(rp, horizon_us=H)) == O.replan(dict(rp, horizon_us=H))
    ar = dict(rp, allreduce_us=1500 + 300 * i)
    assert B.replan(ar) == O.replan(ar)
    # bounded split searches: the same plan
    assert B.replan(dict(rp, bounded_search=1)) == want
    assert B.replan(dict(ar, bounded_search=1)) == O.replan(ar)


def test_full_size_replan_of_the_32_card_shape(B):
    """chm_replan at the size the benchmark times (31 surviving nodes, 6.7e9 splits).  The oracle cannot
    enumerate the deep pipelines, so: every reported pipeline time is recomputed by the oracle from the
    reported cuts; the splits of the 5- and 6-stage pipelines are compared with the oracle's exhaustive best
    split; no single cut of any chosen split can be moved by one layer to a faster split that fits; the
    transfer volume equals the oracle's Kuhn-Munkres optimum on the 31 x 31 fetch matrix; and the chosen
    candidate maximises (H - t_trans) / t_step over the per-dp results, exactly."""
    from fractions import Fraction
    rp = dict(synth.replan32(), allreduce_us=1800)
    L = rp["L"]
    pf, pb = np.cumsum([0] + list(rp["fwd_us"])), np.cumsum([0] + list(rp["bwd_us"]))
    pw = np.cumsum([0] + list(rp["mem_mib"]))
    p0 = O.layout_p0(L, rp["old_pp"])
    held = [(p0[n % rp["old_pp"]], p0[n % rp["old_pp"] + 1]) for n in range(rp["old_dp"] * rp["old_pp"]) if n not in rp["failed_nodes"]]

    def pipeline_time(n, M, cuts):
        b = [0] + cuts + [L]
        if any(pw[b[j + 1]] - pw[b[j]] > rp["mem_cap_mib"] for j in range(n)):
            return None
        return O.makespan_1f1b([int(pf[b[j + 1]] - pf[b[j]]) for j in range(n)], [int(pb[b[j + 1]] - pb[b[j]]) for j in range(n)], M) \
            + (n - 1) * rp["comm_us"]

    whole, stats = B.replan(rp, with_stats=True)
    whole_b, stats_b = B.replan(dict(rp, bounded_search=1), with_stats=True)
    print("replan32 bounded", stats, stats_b, flush=True)
    assert whole_b == whole and stats_b["splits_evaluated"] < stats["splits_evaluated"] == stats["splits_feasible"]
    per_dp = {}
    for dp in range(rp["dp_min"], rp["dp_max"] + 1):
        got = B.replan(dict(rp, dp_min=dp, dp_max=dp))
        print("replan32 dp", dp, got.get("length"), got.get("t_step_us"), got.get("fetch_mib"), flush=True)
        if not got["found"]:
            assert O.integer_partition(len(held), dp, rp["pp_min"], rp["pp_max"]) is None
            continue
        per_dp[dp] = got
        assert got["length"] == O.integer_partition(len(held), dp, rp["pp_min"], rp["pp_max"])
        assert got["micro_batches"] == O.distribute_batch(rp["micro_batches"], got["length"])
        sizes = []
        for n, M, cuts, t in zip(got["length"], got["micro_batches"], got["cuts"], got["pipeline_us"]):
            assert pipeline_time(n, M, cuts) == t
            for i in range(n - 1):                                   # no faster neighbour one layer away
                for delta in (-1, 1):
                    c2 = list(cuts)
                    c2[i] += delta
                    if c2 != sorted(set(c2)) or c2[0] < 1 or c2[-1] > L - 1:
                        continue
                    t2 = pipeline_time(n, M, c2)
                    assert t2 is None or t2 > t or (t2 == t and O.partition_rank(c2) > O.partition_rank(cuts))
            if n <= 6:                                               # the oracle's own exhaustive split
                want_t, want_cuts = O.best_split(rp["fwd_us"], rp["bwd_us"], rp["mem_mib"], None, n, M, rp["mem_cap_mib"])
                assert (want_t + (n - 1) * rp["comm_us"], want_cuts) == (t, cuts)
            b = [0] + cuts + [L]
            sizes += [b[j + 1] - b[j] for j in range(n)]
        assert got["comm_rounds"] == max(sizes)
        assert got["t_step_us"] == max(got["pipeline_us"]) + rp["allreduce_us"] * got["comm_rounds"]
        pos = [(lo, hi) for n, cuts in zip(got["length"], got["cuts"]) for lo, hi in zip([0] + cuts, cuts + [L])]
        fetch = [[O.missing_interval(rp["mem_mib"], lo, hi, hl, hh) for lo, hi in pos] for hl, hh in held]
        assert got["fetch_mib"] == O.min_assignment(fetch)[0]
        assert got["t_trans_us"] == rp["restart_us"] + rp["xfer_us_per_mib"] * got["fetch_mib"]
    whole = B.replan(rp)
    best_dp = max(sorted(per_dp), key=lambda dp: (Fraction(rp["horizon_us"] - per_dp[dp]["t_trans_us"], per_dp[dp]["t_step_us"]), -dp))
    assert whole["n_candidates"] == len(per_dp)
    assert {k: v for k, v in whole.items() if k != "n_candidates"} == {k: v for k, v in per_dp[best_dp].items() if k != "n_candidates"}


def test_replan_argument_checks(B):
    rp = REPLAN[0]
    for key, val in [("dp_min", 0), ("dp_max", 17), ("pp_max", 33), ("micro_batches", 0), ("horizon_us", 0), ("failed_nodes", [1, 1]),
                     ("failed_nodes", [9])]:
        with pytest.raises(B.ChmError) as e:
            B.replan(dict(rp, **{key: val}))
        assert e.value.code == B.ERR_ARG
        with pytest.raises(O.OracleError):
            O.replan(dict(rp, **{key: val}))
    assert B.replan(dict(rp, mem_cap_mib=1)) == O.replan(dict(rp, mem_cap_mib=1)) == {"found": False, "n_candidates": 3}


def test_large_costs_run_in_64_bit(B):
    """layer times of seconds and hundreds of micro-batches: step times beyond 2^31 us, so the library must take
    its 64-bit kernels; every cost and the argmin still match the oracle, and a cost bound beyond 62 bits is
    refused by both sides"""
    rng = np.random.default_rng(31)
    for i, (L, PP, DP, M, failed) in enumerate([(9, 3, 2, 200, [1]), (12, 4, 3, 256, [2, 9]), (10, 5, 2, 150, [7]), (20, 18, 2, 90, [3])]):
        fwd = rng.integers(8_000_000, 12_000_000, L).astype(np.int32)
        bwd = (2 * fwd.astype(np.int64) * rng.uniform(0.9, 1.1, L)).astype(np.int32)
        mem = rng.integers(400, 600, L).astype(np.int32)
        speed = rng.integers(40_000, 600_000, DP * PP).astype(np.uint32)          # 0.6x .. 9x slower nodes
        sc = synth.scenario(L, PP, DP, M, fwd, bwd, mem, failed, 150, int(mem.sum() * 2.5 / PP), speed=speed,
                            horizon_steps=64, reroute_cap=M // 2 + 40, allreduce_us=(0, 5_000_000)[i % 2], transfer_assign=i % 2)
        print("large costs", i, L, PP, DP, M, failed, flush=True)
        o, g = O.Scenario(sc), B.Scenario(sc)
        assert g.families == o.families and g.n_plans == o.n_plans
        n = min(o.n_plans, 20000)
        want = o.score(0, n)
        feasible = want[want != O.INF]
        assert feasible.size and feasible.max() > 2 ** 40          # far beyond what 32-bit step times could give
        got = gpu_scores(B, g, 0, n)
        assert (got == want).all(), np.flatnonzero(got != want)[:10]
        for f in o.families:
            size = f["n_part"] * f["n_reroute"]
            first, count = f["offset"] + size // 2, min(4000, size - size // 2)
            assert (gpu_scores(B, g, first, count) == o.score(first, count)).all()
            width = min(f["n_part"], 300)
            rc_o, best_o, _ = o.search_range(f["strategy"], 0, width)
            rc_g, best_g = g.search_range(f["strategy"], 0, width)
            assert rc_g == rc_o and same_plan(best_g, best_o)
            # a bounded search has nothing to prune with here (the bounds live in the 32-bit kernels): same result
            for mode in (1, 2):
                g.set_bounded_search(mode)
                rc_b, best_b = g.search_range(f["strategy"], 0, width)
                assert rc_b == rc_o and same_plan(best_b, best_o), (mode, best_b, best_o)
            g.set_bounded_search(0)
    huge = synth.scenario(8, 2, 2, 256, np.full(8, 2 ** 31 - 1, np.int32), np.full(8, 2 ** 31 - 1, np.int32), np.ones(8, np.int32),
                          [0], 0, 100, speed=np.full(4, 2 ** 20, np.uint32), horizon_steps=2 ** 31 - 1)
    with pytest.raises(B.ChmError) as e:
        B.Scenario(huge)
    assert e.value.code == B.ERR_OVERFLOW
    with pytest.raises(O.OracleError) as e2:
        O.Scenario(huge)
    assert e2.value.code == O.ERR_OVERFLOW


def test_error_paths_and_degenerate_cases(B):
    import torch
    sc = SMALL[2]
    g = B.Scenario(sc)
    out = torch.empty(4, dtype=torch.int64, device="cuda")
    with pytest.raises(B.ChmError) as e:
        g.score_plans(g.n_plans - 1, 2, out=out)
    assert e.value.code == B.ERR_RANGE
    with pytest.raises(B.ChmError) as e:
        g.search_range(g.families[0]["strategy"], g.families[0]["n_part"], 1)
    assert e.value.code == B.ERR_RANGE
    with pytest.raises(B.ChmError) as e:
        g.decode_plan(g.n_plans)
    assert e.value.code == B.ERR_RANGE
    for key, val in [("L", 0), ("PP", 33), ("failed_nodes", [0, 0]), ("horizon_steps", 0)]:
        with pytest.raises(B.ChmError) as e:
            B.Scenario(dict(sc, **{key: val}))
        assert e.value.code == B.ERR_ARG
    # a stage that lost every peer cannot be rerouted
    un = synth.scenario(8, 4, 2, 8, np.full(8, 10, np.int32), np.full(8, 20, np.int32), np.ones(8, np.int32),
                        [1, 5], 0, 100)
    g2, o2 = B.Scenario(un), O.Scenario(un)
    assert g2.families == o2.families and g2.family(2) is None
    rc, best = g2.search_best(1 << 2)
    assert rc == B.ERR_UNRECOVERABLE == o2.search(1 << 2)[0]
    # nothing fits in memory
    tight = dict(sc, mem_cap_mib=1)
    g3 = B.Scenario(tight)
    rc, best = g3.search_best(7)
    assert rc == B.ERR_NO_FEASIBLE and best["cost"] == B.INFEASIBLE and best["index"] == 2 ** 64 - 1
    assert (gpu_scores(B, g3, 0, g3.n_plans) == B.INFEASIBLE).all()
    # all costs equal -> index 0; equal minima in different workgroups -> the lower index
    flat = synth.scenario(12, 3, 3, 4, np.full(12, 10, np.int32), np.full(12, 20, np.int32), np.ones(12, np.int32),
                          [4], 0, 1000, reconf_us=(0, 0, 0), xfer_us_per_mib=0)
    g4, o4 = B.Scenario(flat), O.Scenario(flat)
    for mask in (1, 2, 4, 7):
        assert same_plan(g4.search_best(mask)[1], o4.search(mask)[1])
    # one micro-batch crosses every stage once, so every partition that fits has the same step time:
    # thousands of equal minima spread over many workgroups, the first feasible index is not 0
    wide = synth.scenario(40, 4, 2, 1, np.full(40, 10, np.int32), np.full(40, 20, np.int32), np.ones(40, np.int32),
                          [], 0, 24, reconf_us=(0, 0, 0), xfer_us_per_mib=0)
    g5, o5 = B.Scenario(wide), O.Scenario(wide)          # C(39,3) = 9139 partitions per family
    costs = o5.score(0, o5.n_plans)
    assert (costs == costs.min()).sum() > 100 and int(np.argmin(costs)) > 0
    for mask in (1, 4, 7):
        lo = 0 if mask != 4 else o5.family(2)["offset"]
        hi = o5.family(0)["n_part"] if mask == 1 else o5.n_plans
        rc, best = g5.search_best(mask)
        assert rc == 0 and best["index"] == lo + int(np.argmin(costs[lo:hi])) and best["cost"] == int(costs[lo:hi].min())
        assert same_plan(best, o5.search(mask)[1])


def test_rank_partitions_and_search_over_explicit_lists(B):
    import torch
    for sc in (synth.config4(), SMALL[3], SMALL[12], SMALL[24], synth.config2()):
        o, g = O.Scenario(sc), B.Scenario(sc)
        for f in o.families:
            k = f["stages"] - 1
            if k == 0:
                continue
            n = 1500
            cuts = synth.random_partitions(77, 5 + f["strategy"], n, sc["L"], k)
            cuts[7] = cuts[3]                                   # duplicates are allowed in a list
            want_ranks = O.partition_rank_batch(cuts)
            d_cuts = torch.from_numpy(cuts).cuda()
            d_ranks = g.rank_partitions(f["strategy"], d_cuts)
            torch.cuda.synchronize()
            assert (d_ranks.cpu().numpy().view(np.uint64) == want_ranks).all()
            # costs of the listed partitions and the first position of their minimum
            if f["n_reroute"] == 1:
                want = o.score_ranks(f["strategy"], want_ranks)
            else:
                want = np.array([o.search_range(f["strategy"], int(r), 1)[1]["cost"] for r in want_ranks[:200]], dtype=np.int64)
                d_ranks, want_ranks = d_ranks[:200].contiguous(), want_ranks[:200]
            costs = torch.empty(len(want), dtype=torch.int64, device="cuda")
            rc, best, pos = g.search_ranks(f["strategy"], d_ranks, costs=costs)
            assert (costs.cpu().numpy() == want).all()
            if (want == O.INF).all():
                assert rc == B.ERR_NO_FEASIBLE
                continue
            assert rc == 0 and pos == int(np.argmin(want)) and best["cost"] == int(want.min())
            rc_o, best_o, _ = o.search_range(f["strategy"], int(want_ranks[pos]), 1)
            assert same_plan(best, best_o)
            # the same list handed over as cut positions
            costs2 = torch.empty(len(want), dtype=torch.int64, device="cuda")
            rc2, best2, pos2 = g.search_cuts(f["strategy"], d_cuts[:len(want)].contiguous(), costs=costs2)
            assert (rc2, pos2) == (rc, pos) and same_plan(best2, best) and torch.equal(costs2, costs)
            # bounded list searches: same winner, same position
            for mode in (1, 2):
                g.set_bounded_search(mode)
                rc3, best3, pos3 = g.search_ranks(f["strategy"], d_ranks)
                rc4, best4, pos4 = g.search_cuts(f["strategy"], d_cuts[:len(want)].contiguous())
                assert (rc3, pos3) == (rc, pos) and same_plan(best3, best), (mode, best3, best)
                assert (rc4, pos4) == (rc, pos) and same_plan(best4, best), (mode, best4, best)
            g.set_bounded_search(0)
    # malformed rows and ranks outside the family
    sc = synth.small_random(2002, L=8, PP=4, DP=2, M=5, n_failed=1, hetero=False)
    g = B.Scenario(sc)
    f = g.family(2)
    assert f["stages"] == 4
    bad = torch.tensor([[3, 2, 5], [0, 1, 2], [1, 2, 200], [1, 2, 3]], dtype=torch.uint8, device="cuda")
    r = g.rank_partitions(f["strategy"], bad).cpu().numpy().view(np.uint64)
    assert (r[:3] == np.uint64(2 ** 64 - 1)).all() and r[3] == 0
    rc, best, pos = g.search_ranks(f["strategy"], torch.tensor([-1, -1], dtype=torch.int64, device="cuda"))
    assert rc == B.ERR_NO_FEASIBLE and best["cost"] == B.INFEASIBLE
    costs = torch.empty(4, dtype=torch.int64, device="cuda")
    rc, best, pos = g.search_cuts(f["strategy"], bad, costs=costs)          # only the last row is a partition
    want = O.Scenario(sc).score_ranks(f["strategy"], [0]) if f["n_reroute"] == 1 else None
    got = costs.cpu().numpy()
    assert (got[:3] == B.INFEASIBLE).all()
    if got[3] == B.INFEASIBLE:
        assert rc == B.ERR_NO_FEASIBLE
    else:
        assert rc == 0 and pos == 3 and best["cuts"] == [1, 2, 3] and best["cost"] == got[3]
        assert want is None or got[3] == want[0]


def test_full_size_config4_explicit_batch(B):
    """2^24 random partitions per strategy: every cost goes through the C-ABI, a seeded sample of
    them is re-scored by the oracle, and the argmin must be the first minimum of the cost array."""
    import torch
    sc = synth.config4(mem_cap_mib=synth.CONFIG4_CAP_30PCT)
    o, g = O.Scenario(sc), B.Scenario(sc)
    n, chunk = 1 << 24, 1 << 18
    rng = np.random.default_rng(9)
    for strategy, k in ((0, 15), (1, 14), (2, 15)):
        d_ranks = torch.empty(n, dtype=torch.int64, device="cuda")
        sample_idx = np.sort(rng.choice(n, 600, replace=False))
        sample_cuts = np.empty((600, k), dtype=np.uint8)
        for c0 in range(0, n, chunk):
            cuts = synth.random_partitions(synth.BASE_SEED + 4, 1000 * strategy + c0 // chunk, chunk, 96, k)
            g.rank_partitions(strategy, torch.from_numpy(cuts).cuda(), out=d_ranks[c0:c0 + chunk])
            sel = (sample_idx >= c0) & (sample_idx < c0 + chunk)
            sample_cuts[sel] = cuts[sample_idx[sel] - c0]
        print("config4 strategy", strategy, "ranks ready", flush=True)
        costs = torch.empty(n, dtype=torch.int64, device="cuda")
        rc, best, pos = g.search_ranks(strategy, d_ranks, costs=costs)
        h = costs.cpu().numpy()
        want_ranks = O.partition_rank_batch(sample_cuts)
        assert (d_ranks.cpu().numpy().view(np.uint64)[sample_idx] == want_ranks).all()
        assert (h[sample_idx] == o.score_ranks(strategy, want_ranks)).all()
        print("config4 strategy", strategy, "infeasible fraction", float((h == B.INFEASIBLE).mean()), flush=True)
        if (h == B.INFEASIBLE).all():
            assert rc == B.ERR_NO_FEASIBLE
            continue
        assert rc == 0 and pos == int(np.argmin(h)) and best["cost"] == int(h.min())
        assert o.plan_cost(strategy, best["cuts"], best["reroute"] if strategy == 2 else None) == best["cost"]
        # the plain scoring entry point gives the same numbers
        again = g.score_ranks(strategy, d_ranks[:100000].contiguous())
        assert torch.equal(again, costs[:100000])
        # and so does the list handed over as cut positions (first 2^22 entries)
        m = 1 << 22
        d_cuts = torch.cat([torch.from_numpy(synth.random_partitions(synth.BASE_SEED + 4, 1000 * strategy + c0 // chunk, chunk, 96, k)).cuda()
                            for c0 in range(0, m, chunk)])
        costs2 = torch.empty(m, dtype=torch.int64, device="cuda")
        rc2, best2, pos2 = g.search_cuts(strategy, d_cuts, costs=costs2)
        assert torch.equal(costs2, costs[:m])
        if not (h[:m] == B.INFEASIBLE).all():
            assert rc2 == 0 and pos2 == int(np.argmin(h[:m])) and best2["cost"] == int(h[:m].min())
        # bounded list searches (no cost store): the same winner and position, by ranks and by cut positions
        g.set_bounded_search(1)
        g.set_timing(True)
        rc3, best3, pos3 = g.search_ranks(strategy, d_ranks)
        fit3 = g.get_timing()["feasible"][strategy]
        rc4, best4, pos4 = g.search_cuts(strategy, d_cuts)
        g.set_bounded_search(0)
        assert (rc3, pos3) == (rc, pos) and same_plan(best3, best)
        assert (rc4, pos4) == (rc2, pos2) and same_plan(best4, best2)
        print("config4 strategy", strategy, "bounded list search evaluated", fit3, "of", int((h != B.INFEASIBLE).sum()), "entries that fit", flush=True)
        assert fit3 <= int((h != B.INFEASIBLE).sum())


def test_full_size_search_config3_and_config5(B):
    """whole spaces of the heterogeneous-rerouting shape (two stages lost a node, 2,380,833 capped
    vectors each) and of a two-failure scenario of the sweep: the winner is re-scored by the oracle
    and must equal the oracle's argmin over the partitions around it."""
    for name, sc in (("config3", synth.config3()), ("config5", synth.config5([9, 13])), ("config5", synth.config5([2, 24]))):
        o, g = O.Scenario(sc), B.Scenario(sc)
        for f in o.families:
            rc, best = g.search_best(1 << f["strategy"])
            print(name, "strategy", f["strategy"], rc, best["index"], best["cost"], flush=True)
            if rc == B.ERR_NO_FEASIBLE:
                assert o.search_range(f["strategy"], 0, min(f["n_part"], 3000))[0] == O.ERR_NO_FEASIBLE
                continue
            rr = best["reroute"] if f["strategy"] == 2 else None
            assert o.plan_cost(f["strategy"], best["cuts"], rr) == best["cost"]
            part = O.partition_rank(best["cuts"])
            width = 60 if f["n_reroute"] > 10 ** 6 else 4000
            lo = max(0, part - width // 2)
            rc_o, best_o, _ = o.search_range(f["strategy"], lo, min(width, f["n_part"] - lo))
            assert rc_o == 0 and same_plan(best, best_o)
        rc_all, best_all = g.search_best(7)
        assert rc_all == 0
        per = [g.search_best(1 << f["strategy"]) for f in o.families]
        want = min((b["cost"], b["index"]) for r, b in per if r == 0)
        assert (best_all["cost"], best_all["index"]) == want


def test_independent_handles_on_concurrent_threads(B):
    """different handles may be used from different threads at the same time (each on a stream of its own):
    loads, exhaustive and bounded searches, cost stores and releases interleave, every result equals the
    single-threaded one"""
    import threading
    import torch
    scs = [synth.small_random(3100 + i, L=14 + i % 5, PP=4 + i % 3, DP=2 + i % 3, M=4 + i) for i in range(8)] + [synth.config1()]
    want = []
    for sc in scs:
        g = B.Scenario(sc)
        want.append((g.search_best(7), g.score_plans(0, min(g.n_plans, 5000)).cpu().numpy()))
        g.close()
    errors = []

    def worker(t):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(6):
                    for i, sc in enumerate(scs):
                        if (i + rep) % 4 != t % 4 and rep % 2:
                            continue
                        g = B.Scenario(sc)
                        g.set_bounded_search((rep + t) % 3)
                        got = g.search_best(7, stream=stream)
                        costs = g.score_plans(0, min(g.n_plans, 5000), stream=stream)
                        stream.synchronize()
                        if got != want[i][0] or not (costs.cpu().numpy() == want[i][1]).all():
                            errors.append((t, rep, i))
                        g.close()
        except Exception as exc:                       # noqa: BLE001 - reported below
            errors.append((t, repr(exc)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(4)]
    for th in threads:
        th.start()
    for th in threads:
        th.join()
    assert not errors, errors[:5]


def _reroute_case(seed, DP, M, cap, failed, L=9, PP=3, hetero=True):
    fwd, bwd, mem = synth.layer_tables(seed, L)
    return synth.scenario(L, PP, DP, M, fwd, bwd, mem, failed, 130, int(mem.sum() * 1.9 / PP),
                          speed=synth.speed_factors(seed, DP, PP) if hetero else None, reroute_cap=cap)


GROUPED = [
    ("p4_cap16_two_stages", _reroute_case(9101, 5, 32, 16, [1, 5])),          # 2 x 3,281 vectors
    ("p5_cap16", _reroute_case(9102, 6, 32, 16, [4])),                        # 39,525
    ("p6_cap16", _reroute_case(9103, 7, 32, 16, [8])),                        # 342,873
    ("p7_cap16_two_stages", _reroute_case(9104, 8, 32, 16, [0, 10])),         # 2 x 2,380,833 (the shape of config 3)
    ("p5_cap8_two_stages", _reroute_case(9105, 6, 16, 8, [2, 9])),            # 2 x 3,195
    ("p6_cap8", _reroute_case(9106, 7, 16, 8, [7])),                          # 15,597
    ("p7_cap8", _reroute_case(9107, 8, 16, 8, [3])),                          # 62,601
    ("p8_cap8", _reroute_case(9108, 9, 16, 8, [13])),                         # 217,701
    ("p6_cap12_run_sweep", _reroute_case(9109, 7, 24, 12, [5])),              # a cap the grouped sweep is not compiled for
    ("p5_cap16_three_stages", _reroute_case(9110, 6, 32, 16, [0, 4, 8])),     # 3 x 39,525: every stage lost a node
    # identical peers: thousands of vectors share the least penalty, the lowest rank among them must come out
    ("p5_cap16_identical_peers", _reroute_case(9111, 6, 32, 16, [4], hetero=False)),
    ("p7_cap8_identical_peers_two_stages", _reroute_case(9112, 8, 16, 8, [1, 11], hetero=False)),
    ("p6_cap12_identical_peers", _reroute_case(9113, 7, 24, 12, [5], hetero=False)),
]


@pytest.mark.parametrize("name", [c[0] for c in GROUPED])
def test_large_reroute_spaces_swept_by_kernels_of_their_own(B, name):
    """more than 4,096 reroute vectors: base pass, the partitions that fit gathered into a list, one sweep launch per
    stage that lost nodes (grouped by shared leading entries where the cap allows), combine; exhaustive and bounded
    against the oracle, with part of the partitions failing the memory filter"""
    sc = dict(GROUPED)[name]
    o, g = O.Scenario(sc), B.Scenario(sc)
    assert g.families == o.families
    f = o.family(2)
    if f is None:
        pytest.skip("rerouting cannot absorb this failure set")
    assert f["n_reroute"] > 4096
    g.set_timing(True)
    rc_o, best_o, _ = o.search_range(2, 0, f["n_part"])
    _, _, fit_o = o.search_range_counted(2, 0, f["n_part"])
    assert 0 < fit_o < f["n_part"]                     # some partitions fit, some do not
    for bounded in (0, 1, 2):
        g.set_bounded_search(bounded)
        rc, best = g.search_best(4)
        assert rc == rc_o == 0 and same_plan(best, best_o), (name, bounded, best, best_o)
        if bounded == 0:
            assert g.get_timing()["feasible"][2] == fit_o
    g.set_bounded_search(0)
    lo, n = f["n_part"] // 4, f["n_part"] // 2
    rc_w, best_w = g.search_range(2, lo, n)
    rc_ow, best_ow, _ = o.search_range(2, lo, n)
    assert rc_w == rc_ow and (rc_w != 0 or same_plan(best_w, best_ow))
    rc_all, best_all = g.search_best(7)
    rc_oa, best_oa = o.search(7)
    assert rc_all == rc_oa == 0 and same_plan(best_all, best_oa)
    g.close()


def test_load_search_and_free_do_not_wait_for_other_streams(B):
    """a handle is loaded, searched and freed while another handle's cost stores are queued on another stream:
    neither the load nor the release waits for the whole device.  (Streams share a few hardware queues, and work
    behind a busy stream's on the same queue does wait for it; so the check is made against several busy
    streams in turn and must hold for at least one: a device-wide wait would fail for all.)"""
    import time
    import torch
    big = B.Scenario(synth.config2())
    f0 = big.family(0)
    count = f0["n_part"]                                 # every plan of the redundant strategy: about a millisecond per call
    out = torch.empty(count, dtype=torch.int64, device="cuda")
    mine = torch.cuda.Stream()
    small = synth.config1()
    g = B.Scenario(small)
    want = g.search_best(7, stream=mine)
    g.close()
    torch.cuda.synchronize()
    loaded, searched, report = 0, 0, []
    for trial in range(6):
        busy = torch.cuda.Stream()
        for _ in range(30):
            big.score_plans(f0["offset"], count, out=out, stream=busy)
        t0 = time.perf_counter()
        g = B.Scenario(small)                            # load and free alone
        g.close()
        ok_load = not busy.query()
        t_load = time.perf_counter() - t0
        g = B.Scenario(small)                            # and with a search in between
        got = g.search_best(7, stream=mine)
        g.close()
        ok_search = not busy.query()
        t_search = time.perf_counter() - t0 - t_load
        assert got == want
        busy.synchronize()
        t_all = time.perf_counter() - t0
        loaded += ok_load
        searched += ok_search
        report.append("%.2f/%.2f/%.1f ms%s" % (t_load * 1e3, t_search * 1e3, t_all * 1e3, "" if ok_load else " (waited)"))
    print("load+free / load+search+free / busy stream drained, per busy stream:", "; ".join(report), flush=True)
    assert loaded >= 1 and searched >= 1
    # the busy handle's own release waits for its own stream only, and its results are intact
    ref = O.Scenario(synth.config2()).score(f0["offset"] + 1000, 64)
    assert (out[1000:1064].cpu().numpy() == ref).all()
    big.close()


REPLAN_TABLES = [
    (synth.replan_case(31, 12, 4, 4, [5, 10, 3, 12, 0], 32, (2, 6), (1, 6)), 5),
    (synth.replan_case(32, 10, 3, 3, [4, 0, 8], 12, (1, 4), (1, 6), act=True), 3),
    (synth.replan_case(33, 14, 2, 6, [7, 1, 10, 4], 24, (1, 4), (2, 8), dist="lognormal"), 4),
    (synth.replan_case(34, 9, 2, 3, [2, 3, 4, 0, 1, 5], 6, (1, 3), (1, 3)), 6),          # down to nothing
]


@pytest.mark.parametrize("i", range(len(REPLAN_TABLES)))
def test_replan_table_for_the_loss_of_one_to_k_nodes(B, i):
    """chm_replan_table: the cached plans for 1 .. k lost nodes (Algorithm 1's loop over failure counts; Planner,
    overhead paragraph) equal the oracle's re-plan of every prefix of the failure order, exhaustive and bounded, and
    equal chm_replan called entry by entry"""
    rp, k = REPLAN_TABLES[i]
    want = [O.replan(dict(rp, failed_nodes=rp["failed_nodes"][:n])) for n in range(1, k + 1)]
    got, stats = B.replan_table(rp, k, with_stats=True)
    assert got == want, (got, want)
    assert B.replan_table(dict(rp, bounded_search=1), k) == want
    assert B.replan_table(dict(rp, allreduce_us=900), k) == [O.replan(dict(rp, allreduce_us=900, failed_nodes=rp["failed_nodes"][:n]))
                                                             for n in range(1, k + 1)]
    assert [B.replan(dict(rp, failed_nodes=rp["failed_nodes"][:n])) for n in range(1, k + 1)] == want
    assert B.replan_table(rp, 0) == []
    with pytest.raises(B.ChmError) as err:
        B.replan_table(rp, len(rp["failed_nodes"]) + 1)
    assert err.value.code == B.ERR_ARG
    # the table searches every (pipeline length, micro-batch count) once: entry by entry the calls search at least as much
    alone = sum(B.replan(dict(rp, failed_nodes=rp["failed_nodes"][:n]), with_stats=True)[1]["splits_scored"] for n in range(1, k + 1))
    assert sum(s["splits_scored"] for s in stats) <= alone
    print("replan table", i, "splits searched", sum(s["splits_scored"] for s in stats), "against", alone, "entry by entry", flush=True)


def test_replan_table_of_the_32_card_shape(B):
    """the table for the loss of 1 .. 3 nodes at the size the benchmark times: every entry equals chm_replan on
    its own (whose first entry the full-size test above checks against the oracle)"""
    rp = dict(synth.replan32(), failed_nodes=synth.replan32()["failed_nodes"] + [13, 20], bounded_search=1)
    table = B.replan_table(rp, 3)
    for n in range(1, 4):
        assert table[n - 1] == B.replan(dict(rp, failed_nodes=rp["failed_nodes"][:n]))
        assert table[n - 1]["found"]
