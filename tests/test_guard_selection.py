"""Which kernels the scenarios of tests/guard_cases.py select (host only: chm_kernel_selection needs no device).
Each pair sits one microsecond (or one MiB) apart on the two sides of a load-time bound; the GPU parity of the
same scenarios is in test_gpu_guards.py."""
import numpy as np
import pytest

from oracle import oracle as O
from tests import guard_cases

CASES = guard_cases.cases()


@pytest.fixture(scope="module")
def B():
    from paper_2508_21613_amd import binding
    binding.lib()
    return binding


@pytest.mark.parametrize("i", range(len(CASES)), ids=[c[0] for c in CASES])
def test_selection_is_on_the_expected_side(B, i):
    name, sc, want = CASES[i]
    sel = B.kernel_selection(sc)
    for key, value in want.items():
        if key == "specialised_any":
            assert any(sel["specialised"]) == value, (name, sel)
        elif key == "sharp_bound":
            used = [sel["sharp_bound"][k] for k in range(3) if sel["specialised"][k]]
            assert used and all(x == value for x in used), (name, sel)
        elif key == "reroute_mul24":
            assert sel[key] == value, (name, sel)
            if sel["present"][2]:
                assert sel["specialised"][2] == value, (name, sel)
        else:
            assert sel[key] == value, (name, key, sel)


def test_pairs_are_neighbours():
    """the two sides of a bound differ by one unit in the bounded quantity and by nothing else"""
    by_name = {c[0]: c[1] for c in CASES}
    for name, sc in by_name.items():
        if not name.endswith("_below"):
            continue
        other = by_name[name[:-6] + "_above"]
        t0 = int(sc["fwd_us"].astype(np.int64).sum() + sc["bwd_us"].astype(np.int64).sum())
        t1 = int(other["fwd_us"].astype(np.int64).sum() + other["bwd_us"].astype(np.int64).sum())
        m0, m1 = int(sc["mem_mib"].astype(np.int64).sum()), int(other["mem_mib"].astype(np.int64).sum())
        a0 = 0 if sc.get("act_mib") is None else int(sc["act_mib"].astype(np.int64).sum())
        a1 = 0 if other.get("act_mib") is None else int(other["act_mib"].astype(np.int64).sum())
        assert sorted([t1 - t0, m1 - m0, a1 - a0]) == [0, 0, 1], name
        assert all(sc[k] == other[k] for k in ("L", "PP", "DP", "M", "failed_nodes", "comm_us"))


@pytest.mark.parametrize("i", range(len(CASES)), ids=[c[0] for c in CASES])
def test_the_oracle_scores_every_plan_of_a_guard_case(i):
    """the oracle works in int64 throughout: the cases are ordinary inputs for it, with some plans that fit"""
    name, sc, _ = CASES[i]
    o = O.Scenario(sc)
    assert o.n_plans <= 200000
    costs = o.score(0, o.n_plans)
    assert (costs != O.INF).any() and (costs > 0).all()
    rc, best = o.search(7)
    assert rc == O.OK and best["index"] == int(np.argmin(costs)) and best["cost"] == int(costs.min())
