"""chm_search_best_static (the entry point that allocates nothing) against chm_search_best, through the C-ABI."""
import pytest

from paper_2508_21613_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2508_21613_amd import binding
    binding.lib()
    return binding


def _both(B, sc, mask=7):
    g = B.Scenario(sc)
    g.set_timing(True)
    want = g.search_best(mask)
    want_t = g.get_timing()
    got = g.search_best_static(mask)
    got_t = g.get_timing()
    again = g.search_best(mask)                       # the handle's own buffers are back in place
    g.close()
    assert got == want and again == want, (got, want, again)
    for key in ("partitions", "evaluations", "feasible", "evaluated"):
        assert got_t[key] == want_t[key], key
    return want


def test_two_calls_in_a_row_the_second_smaller(B):
    # a mid-size space with all three strategies (several tiles and a ragged tail per family), then a smaller one:
    # the array keeps the first call's words, the second call must not see them
    big = synth.small_random(4242, L=26, PP=6, DP=3, M=8, n_failed=1, hetero=False)
    rc_big, best_big = _both(B, big)
    assert rc_big == B.OK and best_big["cost"] < B.INFEASIBLE
    small = synth.config1()
    rc_small, best_small = _both(B, small)
    assert rc_small == B.OK
    from oracle import oracle as O
    for sc, best in ((big, best_big), (small, best_small)):
        rc_o, best_o = O.Scenario(sc).search(7)
        assert rc_o == O.OK and best_o == best


def test_single_strategies_and_heterogeneous_speeds(B):
    sc = synth.small_random(77, L=14, PP=4, DP=4, M=6, n_failed=2, hetero=True, cap=4)
    for mask in (1, 2, 4, 3, 6, 7):
        _both(B, sc, mask)


def test_nothing_fits(B):
    sc = dict(synth.config1(), mem_cap_mib=1)
    g = B.Scenario(sc)
    rc, best = g.search_best_static(7)
    assert rc == B.ERR_NO_FEASIBLE and best["cost"] == B.INFEASIBLE and best["index"] == (1 << 64) - 1
    g.close()


def test_limits_are_errors(B):
    # config 3: 2 x 2,380,833 reroute vectors are swept by kernels of their own, which need scratch per partition
    g = B.Scenario(synth.config3())
    rc, best = g.search_best_static(7)
    assert rc == B.ERR_LIMIT and best["cost"] == B.INFEASIBLE
    rc, best = g.search_best_static(3)                # without the rerouting family the call goes through
    assert (rc, best) == g.search_best(3)
    g.close()
    # costs of tens of seconds per layer leave few index bits in the packed key: 62.9 M partitions are then more chunks
    # than the fixed array has words for
    sc = synth.config2()
    sc = dict(sc, fwd_us=sc["fwd_us"] * 30000, bwd_us=sc["bwd_us"] * 30000)     # 11 index bits: 30,709 chunks
    g = B.Scenario(sc)
    rc, best = g.search_best_static(1)
    assert rc == B.ERR_LIMIT and best["cost"] == B.INFEASIBLE
    g.close()
