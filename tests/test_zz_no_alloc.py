"""The knapsack selection on the library's own fixed device array (the entry point for callers that cannot
allocate) against the entry point that takes a caller workspace: identical op codes, bit for bit, on two
calls in a row, the second on a smaller problem that leaves most of the first call's tables behind."""
import numpy as np
import pytest

import d2ft_inputs as di

pytestmark = pytest.mark.gpu


def both(ks):
    import paper_2504_12471_amd as P
    a = P.d2ft_select_knapsack_static(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    b = P.d2ft_select_knapsack(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    return a, b


def test_static_workspace_matches_caller_workspace_twice():
    import paper_2504_12471_amd as P
    from oracle import d2ft_oracle as orc
    big = di.draw_knapsack_inputs(np.random.default_rng(11), 6, 300, 2, 3, 0.55)
    small = di.draw_knapsack_inputs(np.random.default_rng(12), 2, 48, 1, 2, 0.6)
    for name, ks in (("first call, 6 x 300 items", big), ("second call, 2 x 48 items", small)):
        need = P.d2ft_knapsack_workspace_bytes(ks.score_full.shape[0], ks.score_full.shape[1], ks.cap_full, ks.cap_fwd)
        assert 0 < need <= P.d2ft_knapsack_static_bytes()
        print(f"[no-alloc knapsack] {name}: workspace {need} of {P.d2ft_knapsack_static_bytes()} bytes", flush=True)
        got, want = both(ks)
        assert got.dtype == np.uint8 and got.shape == want.shape
        assert np.array_equal(got, want)
        ref = orc.knapsack_scheduling(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
        assert np.array_equal(got, ref)


def test_static_workspace_rejects_oversized_problem():
    import paper_2504_12471_amd as P
    ks = di.draw_knapsack_inputs(np.random.default_rng(13), 8, 4000, 1, 2, 0.6)
    need = P.d2ft_knapsack_workspace_bytes(8, 4000, ks.cap_full, ks.cap_fwd)
    assert need > P.d2ft_knapsack_static_bytes()
    with pytest.raises(P.D2ftError) as e:
        P.d2ft_select_knapsack_static(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    assert e.value.status == P.binding.ESHAPE
