"""GPU parity of the scenarios of tests/guard_cases.py: one unit below and one unit above every load-time bound
that selects the int32 shape-specialised kernels (and their 24-bit multiplies) over the generic int64 ones.  Every
plan cost and the argmin of every search mode against the oracle (Estimator, eq. (transition): the same recurrence
at the largest magnitudes each kernel family accepts)."""
import numpy as np
import pytest

from oracle import oracle as O
from tests import guard_cases

pytestmark = pytest.mark.gpu

CASES = guard_cases.cases()
KEYS = ("index", "cost", "strategy", "stages", "cuts", "n_affected", "affected_stage", "reroute", "t_step_us", "t_trans_us")


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2508_21613_amd import binding
    binding.lib()
    return binding


def _same(a, b):
    return all(a[k] == b[k] for k in KEYS)


@pytest.mark.parametrize("i", range(len(CASES)), ids=[c[0] for c in CASES])
def test_every_cost_and_every_search_mode(B, i):
    import torch
    name, sc, _ = CASES[i]
    o, g = O.Scenario(sc), B.Scenario(sc)
    assert g.families == o.families and g.n_plans == o.n_plans
    want = o.score(0, o.n_plans)
    got = g.score_plans(0, g.n_plans)
    torch.cuda.synchronize()
    assert (got.cpu().numpy() == want).all(), name
    # a window that starts and ends inside families
    lo, hi = o.n_plans // 7, o.n_plans - o.n_plans // 5
    assert (g.score_plans(lo, hi - lo).cpu().numpy() == want[lo:hi]).all()
    masks = [7] + [1 << f["strategy"] for f in o.families]
    for mask in masks:
        rc_o, best_o = o.search(mask)
        for bounded, compaction in ((0, -1), (0, 0), (0, 1), (1, -1), (2, -1), (2, 1)):
            g.set_bounded_search(bounded)
            g.set_filter_compaction(compaction)
            rc, best = g.search_best(mask)
            assert rc == rc_o and (rc != B.OK or _same(best, best_o)), (name, mask, bounded, compaction, best, best_o)
        g.set_bounded_search(0)
        g.set_filter_compaction(-1)
        rc, best = g.search_best_static(mask)
        assert rc == rc_o and (rc != B.OK or _same(best, best_o)), (name, mask, "static")
    for f in o.families:
        n = f["n_part"]
        for first, count in ((0, n), (n // 3, n - n // 3), (n // 2, max(1, n // 4)), (n - 1, 1)):
            rc_o, best_o, _ = o.search_range(f["strategy"], first, count)
            for bounded in (0, 2):
                g.set_bounded_search(bounded)
                rc, best = g.search_range(f["strategy"], first, count)
                assert rc == rc_o and (rc != B.OK or _same(best, best_o)), (name, f["strategy"], first, count, bounded)
        g.set_bounded_search(0)
        # explicit lists: every partition once, in a seeded order
        order = np.random.default_rng(i).permutation(n).astype(np.uint64)
        d_ranks = torch.from_numpy(order.view(np.int64)).cuda()
        costs = torch.empty(n, dtype=torch.int64, device="cuda")
        rc, best, pos = g.search_ranks(f["strategy"], d_ranks, costs=costs)
        rc_o, best_o = o.search(1 << f["strategy"])
        assert rc == rc_o
        if rc == B.OK:
            # equal costs in a list go to the lowest list position: the oracle's best plan of every single partition,
            # first minimum in list order
            per = [o.search_range(f["strategy"], int(r), 1) for r in order]
            per_cost = np.array([p[1]["cost"] if p[0] == O.OK else O.INF for p in per])
            assert best["cost"] == best_o["cost"] and pos == int(np.argmin(per_cost)) and _same(best, per[pos][1])
        if f["n_reroute"] == 1:
            assert (costs.cpu().numpy() == o.score_ranks(f["strategy"], order)).all()
            cuts = np.array([O.partition_unrank(sc["L"], f["stages"] - 1, int(r)) for r in order], dtype=np.uint8).reshape(n, f["stages"] - 1)
            costs2 = torch.empty(n, dtype=torch.int64, device="cuda")
            rc2, best2, pos2 = g.search_cuts(f["strategy"], torch.from_numpy(cuts).cuda(), costs=costs2)
            assert (rc2, pos2) == (rc, pos) and torch.equal(costs, costs2)
            for bounded in (1, 2):
                g.set_bounded_search(bounded)
                rc3, best3, pos3 = g.search_ranks(f["strategy"], d_ranks)
                assert (rc3, pos3) == (rc, pos) and (rc != B.OK or _same(best3, best))
            g.set_bounded_search(0)
    g.close()
