"""Argmin parity over WHOLE plan spaces: chm_search_best (exhaustive and bounded) against the CPU oracle's
exhaustive argmin stored in tests/golden/full_space.json (written by tests/golden/make_full_space.py, which
calls only the oracle): configs 1, 2 and 3 and failure sets of config 5, per strategy and over all
strategies, with the number of partitions that pass the memory filter.  Config 4's explicit lists are
checked cost by cost against the oracle on the fly (first 2^20 entries per strategy).

Algorithm 1, get_execution_plan: the argmin over all candidates; Planner, overhead paragraph: the plan
cache over failure sets.
"""
import json
import os
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from oracle import oracle as O
from paper_2508_21613_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "golden"))
import make_full_space as MFS                          # noqa: E402  (seeded case -> scenario; oracle only)

pytestmark = pytest.mark.gpu

with open(os.path.join(HERE, "golden", "full_space.json")) as _fh:
    GOLD = json.load(_fh)["cases"]

KEYS = ("index", "cost", "strategy", "stages", "cuts", "n_affected", "affected_stage", "reroute", "t_step_us", "t_trans_us")


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2508_21613_amd import binding
    binding.lib()
    return binding


def _same(got, want):
    return all(got[k] == want[k] for k in KEYS)


def _check(B, g, mask, want_best, label):
    rc, best = g.search_best(mask)
    if want_best is None:
        assert rc == B.ERR_NO_FEASIBLE and best["cost"] == B.INFEASIBLE, label
    else:
        assert rc == B.OK and _same(best, want_best), (label, best, want_best)
    return g.get_timing()


@pytest.mark.parametrize("name", sorted(GOLD))
def test_whole_space_argmin_equals_the_oracle(B, name):
    rec = GOLD[name]
    sc = MFS.case_scenario(name)
    assert sc["failed_nodes"] == rec["failed_nodes"]
    g = B.Scenario(sc)
    g.set_timing(True)
    assert [(f["strategy"], f["stages"], f["n_part"], f["n_reroute"]) for f in g.families] == \
           [(f["strategy"], f["stages"], f["n_part"], f["n_reroute"]) for f in rec["families"]]
    all_mask = sum(1 << f["strategy"] for f in rec["families"])
    for bounded in (0, 1, 2):
        g.set_bounded_search(bounded)
        t = _check(B, g, all_mask, rec["best"], (name, "all", bounded))
        if bounded == 0:
            # every partition of every family was looked at, and exactly the oracle's count passed the memory filter
            for f in rec["families"]:
                assert t["partitions"][f["strategy"]] == f["n_part"]
                assert t["feasible"][f["strategy"]] == f["feasible"], (name, f["strategy"])
                assert t["evaluated"][f["strategy"]] == f["feasible"]
        for f in rec["families"]:
            t = _check(B, g, 1 << f["strategy"], f["best"], (name, f["strategy"], bounded))
            if bounded == 0:
                assert t["feasible"][f["strategy"]] == f["feasible"]
            else:
                # a bounded search looks at no more partitions than fit, and never loses the winner
                assert t["evaluated"][f["strategy"]] <= f["feasible"]
    # the search that allocates nothing, where its limits allow it
    g.set_bounded_search(0)
    rc, best = g.search_best_static(all_mask)
    if rc != B.ERR_LIMIT:
        assert (rc == B.OK and _same(best, rec["best"])) if rec["best"] is not None else rc == B.ERR_NO_FEASIBLE
    g.close()


def _oracle_costs_threaded(sc, strategy, ranks, threads=16):
    """oracle cost of every rank; the oracle is called from several host threads on handles of their own
    (plain C calls release the interpreter lock)"""
    parts = np.array_split(ranks, threads * 4)

    def work(chunk):
        o = O.Scenario(sc)
        out = o.score_ranks(strategy, chunk)
        o.close()
        return out

    with ThreadPoolExecutor(max_workers=threads) as pool:
        return np.concatenate(list(pool.map(work, parts)))


@pytest.mark.parametrize("strategy,k", [(0, 15), (1, 14), (2, 15)])
def test_config4_first_2_20_entries_cost_by_cost(B, strategy, k):
    """the first 2^20 random partitions of config 4's list of each strategy: every cost and the argmin against
    the oracle (the whole 2^24 list is covered by samples in test_full_size_config4_explicit_batch)"""
    import torch
    sc = synth.config4(mem_cap_mib=synth.CONFIG4_CAP_30PCT)
    g = B.Scenario(sc)
    n, chunk = 1 << 20, 1 << 18
    cuts = np.concatenate([synth.random_partitions(synth.BASE_SEED + 4, 1000 * strategy + c0 // chunk, chunk, 96, k)
                           for c0 in range(0, n, chunk)])
    ranks = O.partition_rank_batch(cuts)
    if O.Scenario(sc).family(strategy)["n_reroute"] != 1:
        pytest.skip("explicit scoring has no reroute argument")
    want = _oracle_costs_threaded(sc, strategy, ranks)
    d_cuts = torch.from_numpy(cuts).cuda()
    costs = torch.empty(n, dtype=torch.int64, device="cuda")
    rc, best, pos = g.search_cuts(strategy, d_cuts, costs=costs)
    got = costs.cpu().numpy()
    assert (got == want).all(), int((got != want).sum())
    if (want == O.INF).all():
        assert rc == B.ERR_NO_FEASIBLE
    else:
        assert rc == B.OK and pos == int(np.argmin(want)) and best["cost"] == int(want.min())
        assert best["cuts"] == [int(x) for x in cuts[pos]]
    d_ranks = torch.from_numpy(ranks.view(np.int64)).cuda()
    for bounded in (0, 1):
        g.set_bounded_search(bounded)
        rc2, best2, pos2 = g.search_ranks(strategy, d_ranks)
        rc3, best3, pos3 = g.search_cuts(strategy, d_cuts)
        assert (rc2, pos2) == (rc, pos) and (rc3, pos3) == (rc, pos)
        if rc == B.OK:
            assert _same(best2, best) and _same(best3, best)
    g.close()


def test_batch_search_equals_the_oracle(B):
    """chm_search_best_batch over every stored case at once (one wait for the whole batch): exhaustive and bounded,
    all strategies and each strategy alone"""
    names = sorted(GOLD)
    gs = [B.Scenario(MFS.case_scenario(n)) for n in names]
    for bounded in (0, 1, 2):
        for g in gs:
            g.set_bounded_search(bounded)
        for mask in (7, 1, 2, 4):
            res = B.search_best_batch(gs, mask)
            assert len(res) == len(names)
            for name, (rc, best) in zip(names, res):
                fams = [f for f in GOLD[name]["families"] if mask & (1 << f["strategy"])]
                if not fams:
                    assert rc == B.ERR_UNRECOVERABLE, (name, mask)
                    continue
                want = MFS.best_of_families(fams)
                if want is None:
                    assert rc == B.ERR_NO_FEASIBLE and best["cost"] == B.INFEASIBLE, (name, mask)
                else:
                    assert rc == B.OK and _same(best, want), (name, mask, bounded, best, want)
    # the handles stay usable one by one, and the call checks its arguments
    for g in gs:
        g.set_bounded_search(0)
    rc, best = gs[0].search_best(7)
    assert rc == B.OK and _same(best, GOLD[names[0]]["best"])
    assert B.search_best_batch([], 7) == []
    with pytest.raises(B.ChmError) as err:
        B.search_best_batch([gs[0], gs[1], gs[0]], 7)
    assert err.value.code == B.ERR_ARG
    for g in gs:
        g.close()


def test_all_528_failure_sets_of_config5(B):
    """the whole failure sweep as the benchmark runs it (one batched call over all 32 single and 496 double failures):
    the exhaustive and the bounded sweep return the same plans, every winner re-scored by the oracle from its cuts and
    reroute vectors has the cost the library reports (and decodes to the index it reports), no plan of the oracle's
    window around it is better, and the 50 failure sets with a stored whole-space result equal it"""
    sets = synth.config5_failure_sets()
    scs = [synth.config5(fs) for fs in sets]
    gs = [B.Scenario(sc) for sc in scs]
    plans = B.search_best_batch(gs, 7)
    for g in gs:
        g.set_bounded_search(1)
    bounded = B.search_best_batch(gs, 7)
    assert len(plans) == 528
    pinned = 0
    for fs, sc, (rc, best), (rc_b, best_b) in zip(sets, scs, plans, bounded):
        assert rc == B.OK and rc_b == B.OK and _same(best, best_b), (fs, best, best_b)
        o = O.Scenario(sc)
        rr = best["reroute"] if best["strategy"] == 2 else None
        assert o.plan_cost(best["strategy"], best["cuts"], rr) == best["cost"], fs
        assert _same(o.decode(best["index"]), best) or o.decode(best["index"])["cuts"] == best["cuts"], fs
        f = o.family(best["strategy"])
        part = O.partition_rank(best["cuts"])
        lo = max(0, part - 150)
        rc_o, best_o, _ = o.search_range(best["strategy"], lo, min(300, f["n_part"] - lo))
        assert rc_o == O.OK and _same(best_o, best), (fs, best_o, best)
        name = "config5:" + ",".join(str(x) for x in fs)
        if name in GOLD:
            assert _same(best, GOLD[name]["best"]), name
            pinned += 1
        o.close()
    assert pinned == 50
    for g in gs:
        g.close()


_MORE = os.path.join(HERE, "golden", "full_space_more.json")
if os.path.exists(_MORE):
    with open(_MORE) as _fh:
        GOLD_MORE = json.load(_fh)["cases"]
else:
    GOLD_MORE = {}


def test_further_double_failures_of_config5(B):
    """tests/golden/full_space_more.json (make_full_space.py --more): the oracle's whole-space argmin of further seeded
    double failures of config 5, as slim records: winner per strategy and overall (index, cost, cuts) and fitting
    partitions, against the exhaustive and the bounded batched search"""
    if not GOLD_MORE:
        pytest.skip("no further cases stored")
    names = sorted(GOLD_MORE)
    gs = [B.Scenario(MFS.case_scenario(n)) for n in names]
    for g in gs:
        g.set_timing(True)

    def same(best, want):
        return all(best[k] == want[k] for k in ("index", "cost", "strategy", "cuts"))

    for bounded in (0, 1):
        for g in gs:
            g.set_bounded_search(bounded)
        for mask in (7, 1, 2, 4):
            res = B.search_best_batch(gs, mask)
            for name, g, (rc, best) in zip(names, gs, res):
                rec = GOLD_MORE[name]
                fams = [f for f in rec["families"] if mask & (1 << f["strategy"])]
                if not fams:
                    assert rc == B.ERR_UNRECOVERABLE, (name, mask)
                    continue
                want = MFS.best_of_families(fams)
                if want is None:
                    assert rc == B.ERR_NO_FEASIBLE, (name, mask)
                    continue
                assert rc == B.OK and same(best, want), (name, mask, bounded, best, want)
                if bounded == 0:
                    t = g.get_timing()
                    for f in fams:
                        assert t["feasible"][f["strategy"]] == f["feasible"], (name, f["strategy"])
    for g in gs:
        g.close()
