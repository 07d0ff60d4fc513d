"""Seeded random small scenarios (shapes, failure sets, caps, speed factors, activation memory, assignment,
communication rounds and time scales drawn from the seed): every plan cost and the argmin of every search entry point
against the oracle.  A fixed slice of a much longer sweep that was run once over ten thousand seeds."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2508_21613_amd import synth

pytestmark = pytest.mark.gpu

KEYS = ("index", "cost", "strategy", "stages", "cuts", "n_affected", "affected_stage", "reroute", "t_step_us", "t_trans_us")


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2508_21613_amd import binding
    binding.lib()
    return binding


def _scenario(seed):
    r = synth.randint(seed, 99, 10, 0, 1 << 30)
    PP = 1 + int(r[0] % 10)
    L = PP + int(r[1] % 9)
    DP = 1 + int(r[2] % 6)
    M = 1 + int(r[3] % 20)
    nf = min(int(r[4] % 5), DP * PP)
    cap = [None, 0, 2, 3, 5, 8, 16][int(r[5] % 7)]
    sc = synth.small_random(seed, L=L, PP=PP, DP=DP, M=M, n_failed=nf, hetero=bool(r[6] % 2), cap=cap)
    if r[7] % 3 == 0:
        sc = synth.with_activations(sc, seed)
    if r[7] % 4 == 0:
        sc = dict(sc, transfer_assign=1)
    if r[7] % 5 == 0:
        sc = dict(sc, allreduce_us=100 + int(r[8] % 900))
    if r[9] % 7 == 0:                                  # near or beyond the bounds of the int32 kernels
        sc = dict(sc, fwd_us=sc["fwd_us"] * 3000, bwd_us=sc["bwd_us"] * 3000)
    return sc


@pytest.mark.parametrize("block", range(8))
def test_random_scenarios(B, block):
    checked = 0
    for seed in range(50001 + 60 * block, 50001 + 60 * (block + 1)):
        sc = _scenario(seed)
        try:
            o = O.Scenario(sc)
        except O.OracleError as e:
            with pytest.raises(B.ChmError) as err:
                B.Scenario(sc)
            assert err.value.code == e.code, seed
            continue
        g = B.Scenario(sc)
        assert g.families == o.families and g.n_plans == o.n_plans, seed
        if o.n_plans == 0 or o.n_plans > 300000:
            g.close()
            continue
        checked += 1
        want = o.score(0, o.n_plans)
        assert (g.score_plans(0, g.n_plans).cpu().numpy() == want).all(), seed
        for mask in [7] + [1 << f["strategy"] for f in o.families]:
            rc_o, best_o = o.search(mask)
            for bounded in (0, 1, 2):
                g.set_bounded_search(bounded)
                rc, best = g.search_best(mask)
                assert rc == rc_o and (rc != 0 or all(best[k] == best_o[k] for k in KEYS)), (seed, mask, bounded, best, best_o)
            g.set_bounded_search(0)
            rc, best = g.search_best_static(mask)
            assert rc == B.ERR_LIMIT or (rc == rc_o and (rc != 0 or all(best[k] == best_o[k] for k in KEYS))), (seed, mask)
            (rc, best), = B.search_best_batch([g], mask)
            assert rc == rc_o and (rc != 0 or all(best[k] == best_o[k] for k in KEYS)), (seed, mask)
        g.close()
    assert checked >= 30
