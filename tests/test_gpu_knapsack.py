"""GPU parity of d2ft_select_knapsack against the oracle's Alg. 1 / Alg. 2: bit-exact codes."""
import numpy as np
import pytest

import d2ft_inputs as di
from oracle import d2ft_oracle as orc

pytestmark = pytest.mark.gpu


def gpu_select(ks):
    import paper_2504_12471_amd as P
    return P.d2ft_select_knapsack(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)


def oracle_select(ks):
    return orc.knapsack_scheduling(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)


def test_share_of_vit_b16_selection():
    """48 heads of one device, costs fwd 1 / full 3, capacity 60% of all-full."""
    ks = di.draw_knapsack_inputs(np.random.default_rng(0), 1, 48, 1, 2, 0.6)
    got, ref = gpu_select(ks), oracle_select(ks)
    assert got.dtype == np.uint8 and np.array_equal(got, ref)
    assert (got == di.OP_FULL).sum() == 28


@pytest.mark.parametrize("seed", range(8))
def test_random_problems_bit_exact(seed):
    rng = np.random.default_rng(100 + seed)
    K, n = int(rng.integers(1, 7)), int(rng.integers(1, 40))
    ks = di.KnapsackInputs(
        score_full=rng.random((K, n)), score_fwd=rng.random((K, n)),
        cost_fwd=rng.integers(1, 4, K).astype(np.int32), cost_bwd=rng.integers(0, 5, K).astype(np.int32),
        cap_full=rng.integers(0, 60, K).astype(np.int32), cap_fwd=rng.integers(0, 30, K).astype(np.int32))
    assert np.array_equal(gpu_select(ks), oracle_select(ks))


def test_many_items_wide_capacity_and_ties():
    rng = np.random.default_rng(7)
    K, n = 3, 300
    # scores on a coarse grid: many equal sums, so the strict-change rule decides
    ks = di.KnapsackInputs(
        score_full=rng.integers(0, 4, (K, n)).astype(np.float64) * 0.25, score_fwd=rng.integers(-1, 3, (K, n)) * 0.5,
        cost_fwd=np.array([1, 2, 3], np.int32), cost_bwd=np.array([2, 0, 4], np.int32),
        cap_full=np.array([700, 90, 0], np.int32), cap_fwd=np.array([33, 400, 5], np.int32))
    assert np.array_equal(gpu_select(ks), oracle_select(ks))


def test_micro_batch_schedule_shape():
    """The paper's own use: per subnet, N = 5 micro-batches, 3 p_f + 2 p_s budget (Sec. III-B)."""
    rng = np.random.default_rng(11)
    K, n = 72, 5
    ks = di.KnapsackInputs(rng.random((K, n)), rng.random((K, n)), np.full(K, 2, np.int32), np.full(K, 3, np.int32),
                           np.full(K, 15, np.int32), np.full(K, 0, np.int32))
    got = gpu_select(ks)
    assert np.array_equal(got, oracle_select(ks))
    assert np.all((got == di.OP_FULL).sum(axis=1) == 3) and np.all((got == di.OP_SKIP).sum(axis=1) == 2)
