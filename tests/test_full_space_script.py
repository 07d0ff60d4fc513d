"""The script that writes tests/golden/full_space.json (tests/golden/make_full_space.py): its sharded sweep of
the oracle must equal the oracle's own single-pass exhaustive search, first minimum included."""
import json
import os
import sys

import numpy as np

from oracle import oracle as O
from paper_2508_21613_amd import synth

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "golden"))
import make_full_space as MFS                          # noqa: E402

KEYS = ("index", "cost", "strategy", "stages", "cuts", "n_affected", "affected_stage", "reroute", "t_step_us", "t_trans_us")


def _same(a, b):
    return all(a[k] == b[k] for k in KEYS)


def test_config1_equals_the_oracle_search_and_the_stored_record():
    rec = MFS.full_space(["config1"], workers=2, chunk_parts=97)["config1"]
    o = O.Scenario(synth.config1())
    rc, best = o.search(7)
    assert rc == O.OK and _same(rec["best"], best)
    for f in rec["families"]:
        rc, b = o.search(1 << f["strategy"])
        assert rc == O.OK and _same(f["best"], b)
        costs = o.score(o.family(f["strategy"])["offset"], f["n_part"] * f["n_reroute"])
        assert f["feasible"] == int((costs.reshape(f["n_part"], f["n_reroute"])[:, 0] != O.INF).sum())
    with open(os.path.join(HERE, "golden", "full_space.json")) as fh:
        stored = json.load(fh)["cases"]["config1"]
    assert json.loads(json.dumps(rec)) == stored


def test_sub_ranges_merge_to_the_first_minimum_among_ties():
    # identical layers: mirrored and shifted partitions tie in cost, so the first minimum is decided by the order
    # in which sub-ranges are merged; every chunk size must give the plan of the single pass
    # (no transfer or restart cost: four partitions of the re-partition strategy and two rerouting plans share the
    # lowest cost)
    L = 11
    sc = synth.scenario(L, 3, 3, 4, np.full(L, 1000, np.int32), np.full(L, 2000, np.int32), np.full(L, 100, np.int32),
                        [4], 100, 700, xfer_us_per_mib=0, reconf_us=(0, 0, 0))
    o = O.Scenario(sc)
    rc, want = o.search(7)
    assert rc == O.OK
    real_case = MFS.case_scenario
    MFS.case_scenario = lambda name: sc if name == "tie" else real_case(name)
    try:
        for chunk in (1, 2, 3, 5, 7, 1000):
            rec = MFS.full_space(["tie"], workers=1, chunk_parts=chunk)["tie"]
            assert _same(rec["best"], want), chunk
            for f in rec["families"]:
                rc, b = o.search(1 << f["strategy"])
                assert (f["best"] is None and rc == O.ERR_NO_FEASIBLE) or _same(f["best"], b)
    finally:
        MFS.case_scenario = real_case
    # the ties are real, inside the winner's strategy and across strategies
    costs = o.score(0, o.n_plans)
    assert int(np.argmin(costs)) == want["index"]
    tied = np.flatnonzero(costs == want["cost"])
    f = o.family(want["strategy"])
    assert int((tied < f["offset"] + f["n_part"] * f["n_reroute"]).sum()) >= 2 and int(tied.max()) >= f["offset"] + f["n_part"] * f["n_reroute"]


def test_stored_records_are_consistent():
    with open(os.path.join(HERE, "golden", "full_space.json")) as fh:
        cases = json.load(fh)["cases"]
    for name, rec in cases.items():
        o = O.Scenario(MFS.case_scenario(name))
        assert [(f["strategy"], f["n_part"], f["n_reroute"]) for f in o.families] == \
               [(f["strategy"], f["n_part"], f["n_reroute"]) for f in rec["families"]], name
        assert rec["best"] == MFS.best_of_families(rec["families"])
        for f in rec["families"]:
            assert 0 <= f["feasible"] <= f["n_part"] and (f["best"] is None) == (f["feasible"] == 0)
            if f["best"] is not None:
                # the stored winner re-scored on its own: cost, step and transition time
                b = f["best"]
                assert o.plan_cost(f["strategy"], b["cuts"], b["reroute"] if f["strategy"] == 2 else None) == b["cost"]
                assert o.decode(b["index"])["cuts"] == b["cuts"]
                assert b["cost"] == sc_horizon(name) * b["t_step_us"] + b["t_trans_us"]


def test_golden_file_covers_what_it_should():
    with open(os.path.join(HERE, "golden", "full_space.json")) as fh:
        GOLD = json.load(fh)["cases"]
    names = set(GOLD)
    assert {"config1", "config2", "config3"} <= names
    singles = [n for n in names if n.startswith("config5:") and "," not in n]
    doubles = [n for n in names if n.startswith("config5:") and "," in n]
    assert len(singles) == 32 and len(singles) + len(doubles) >= 48
    for n in names:
        assert len(GOLD[n]["families"]) >= 1 and all("feasible" in f for f in GOLD[n]["families"])


def sc_horizon(name):
    return MFS.case_scenario(name)["horizon_steps"]


def test_further_stored_records_are_consistent():
    """full_space_more.json (slim records of further double failures of config 5): every stored winner decodes to the
    stored cuts and cost, the overall winner is the first minimum over the strategies, and none of the cases is one
    of the main file's"""
    path = os.path.join(HERE, "golden", "full_space_more.json")
    if not os.path.exists(path):
        return
    with open(path) as fh:
        cases = json.load(fh)["cases"]
    with open(os.path.join(HERE, "golden", "full_space.json")) as fh:
        main = json.load(fh)["cases"]
    wanted = {"config5:%d,%d" % (a, b) for a, b in MFS.config5_more_doubles(len(cases))}
    assert set(cases) <= {"config5:%d,%d" % (a, b) for a, b in MFS.config5_more_doubles(400)} and not set(cases) & set(main)
    assert len(cases) < 8 or len(set(cases) & wanted) >= len(cases) - 8      # (a run in progress may be a few cases ahead)
    for name, rec in cases.items():
        o = O.Scenario(MFS.case_scenario(name))
        assert [(f["strategy"], f["n_part"], f["n_reroute"]) for f in o.families] == \
               [(f["strategy"], f["n_part"], f["n_reroute"]) for f in rec["families"]], name
        assert rec["best"] == MFS.best_of_families(rec["families"])
        for f in rec["families"]:
            assert 0 <= f["feasible"] <= f["n_part"] and (f["best"] is None) == (f["feasible"] == 0)
            if f["best"] is not None:
                d = o.decode(f["best"]["index"])
                assert d["cuts"] == f["best"]["cuts"] and d["cost"] == f["best"]["cost"] and d["strategy"] == f["strategy"]
