"""Pins for the oracle's head compaction, bi-level knapsack and cost rules (no GPU)."""
import itertools
import os

import numpy as np
import pytest

import d2ft_inputs as di
from oracle import d2ft_oracle as orc

FULL, FWD, SKIP = di.OP_FULL, di.OP_FWD, di.OP_SKIP
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------
# compaction
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("H", [1, 2, 3, 4, 5, 6])
def test_compaction_all_masks(H):
    for ops in itertools.product((FULL, FWD, SKIP), repeat=H):
        live, n_full, n_live = orc.compact_heads(ops)
        want_full = sorted(h for h in range(H) if ops[h] == FULL)
        want_fwd = sorted(h for h in range(H) if ops[h] == FWD)
        assert live == want_full + want_fwd
        assert n_full == len(want_full) and n_live == len(want_full) + len(want_fwd)


def test_compaction_rejects_bad_code():
    with pytest.raises(ValueError):
        orc.compact_heads([1, 0, 3])


# ---------------------------------------------------------------------------
# DPSearching against brute force and closed forms
# ---------------------------------------------------------------------------
def brute_force(scores, weight, cap):
    """Best subset value and the set(s) reaching it, by enumeration."""
    n = len(scores)
    best, best_sets = 0.0, [()]
    for r in range(1, n + 1):
        if r * weight > cap:
            break
        for comb in itertools.combinations(range(n), r):
            v = float(sum(scores[i] for i in comb))
            if v > best + 1e-12:
                best, best_sets = v, [comb]
            elif abs(v - best) <= 1e-12:
                best_sets.append(comb)
    return best, best_sets


@pytest.mark.parametrize("seed", range(12))
def test_dp_equals_brute_force(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 13))
    weight = int(rng.integers(1, 5))
    cap = int(rng.integers(0, weight * n + 3))
    scores = rng.random(n)
    sel = orc.dp_searching(scores, weight, cap)
    chosen = tuple(i for i in range(n) if sel[i])
    best, best_sets = brute_force(scores, weight, cap)
    assert len(chosen) * weight <= cap
    assert abs(sum(scores[i] for i in chosen) - best) < 1e-12
    assert len(best_sets) == 1 and chosen == best_sets[0]     # U(0,1) scores: unique optimum


@pytest.mark.parametrize("n,weight,cap", [(10, 3, 17), (48, 3, 86), (48, 1, 2), (7, 2, 100), (5, 4, 3)])
def test_equal_weights_select_top_k(n, weight, cap):
    """With one common weight the optimum is the floor(cap/weight) best positive scores."""
    rng = np.random.default_rng(n * 100 + cap)
    scores = rng.random(n) + 0.01
    sel = orc.dp_searching(scores, weight, cap)
    k = min(n, cap // weight)
    want = set(np.argsort(-scores)[:k].tolist())
    assert set(i for i in range(n) if sel[i]) == want


def test_nonpositive_scores_are_never_taken():
    sel = orc.dp_searching([0.0, -1.0, 0.5, 0.0], 1, 4)
    assert sel == [0, 0, 1, 0]


def test_zero_capacity_and_oversized_weight():
    assert orc.dp_searching([0.3, 0.9], 1, 0) == [0, 0]
    assert orc.dp_searching([0.3, 0.9], 5, 4) == [0, 0]


def test_ties_follow_strict_change_rule():
    # Equal scores: the table value changes at item i only where a new item fits,
    # so the first floor(cap/weight) items by index are kept (tie behaviour is
    # fixed by Alg. 2's "differs from the row above" test alone: parity unpinned
    # beyond this self-consistency).
    assert orc.dp_searching([1.0, 1.0, 1.0, 1.0], 1, 2) == [1, 1, 0, 0]


# ---------------------------------------------------------------------------
# KnapsackScheduling (merge rule, capacities, balance)
# ---------------------------------------------------------------------------
def test_merge_truth_table():
    # item 0: both -> p_f ; item 1: only p_f ; item 2: only p_o ; item 3: neither
    score_full = np.array([[0.9, 0.8, 0.1, 0.2]])
    score_fwd = np.array([[0.9, 0.1, 0.8, 0.2]])
    t = orc.knapsack_scheduling(score_full, score_fwd, [1], [2], [6], [2])
    assert t.tolist() == [[FULL, FULL, FWD, SKIP]]


@pytest.mark.parametrize("seed", range(6))
def test_schedule_respects_capacities(seed):
    rng = np.random.default_rng(seed)
    K, n = 4, 11
    cf = rng.integers(1, 3, K)
    cb = rng.integers(0, 4, K)
    capf = rng.integers(0, 20, K)
    capo = rng.integers(0, 8, K)
    sf, so = rng.random((K, n)), rng.random((K, n))
    t = orc.knapsack_scheduling(sf, so, cf, cb, capf, capo)
    assert set(np.unique(t)).issubset({FULL, FWD, SKIP})
    for k in range(K):
        # stage-wise selections, recomputed independently by brute force
        _, sets_f = brute_force(sf[k], int(cf[k] + cb[k]), int(capf[k]))
        _, sets_o = brute_force(so[k], int(cf[k]), int(capo[k]))
        full = set(sets_f[0]); fwd = set(sets_o[0]) - full
        assert set(np.where(t[k] == FULL)[0].tolist()) == full
        assert set(np.where(t[k] == FWD)[0].tolist()) == fwd
        cost = len(full) * int(cf[k] + cb[k]) + len(fwd) * int(cf[k])
        assert cost <= int(capf[k]) + int(capo[k])


def test_equal_costs_and_capacities_balance_every_subnet():
    """Same costs and capacities on every subnet: every subnet runs the same number of
    p_f and of p_f+p_o items, i.e. workload variance 0 (Sec. III-B, workload-variance table)."""
    rng = np.random.default_rng(3)
    K, n = 9, 5
    sf, so = rng.random((K, n)), rng.random((K, n))
    t = orc.knapsack_scheduling(sf, so, [2] * K, [3] * K, [15] * K, [4] * K)
    n_full = (t == FULL).sum(axis=1)
    assert np.all(n_full == 3)
    load = (t == FULL).sum(axis=1) * 5 + (t == FWD).sum(axis=1) * 2
    # p_o picks 2 items per subnet; those that coincide with p_f items merge into p_f
    assert np.all((t == FWD).sum(axis=1) <= 2)
    assert np.all(load <= 15 + 4)


def test_max_scaler_single_stage_picks_the_same_full_set():
    """Sec. IV-B: scaling forward scores below every backward score makes a single
    knapsack agree with the bi-level outer problem on the p_f set."""
    rng = np.random.default_rng(5)
    n, cf, cb, cap = 8, 1, 2, 12
    sf, so = rng.random(n) + 1.0, rng.random(n) * 1e-6
    t = orc.knapsack_scheduling(sf[None], so[None], [cf], [cb], [cap], [0])
    full = set(np.where(t[0] == FULL)[0].tolist())
    # single-stage multiple-choice optimum by enumeration over {skip, fwd, full}^n
    best, best_assign = -1.0, None
    for assign in itertools.product((0, 1, 2), repeat=n):
        cost = sum((cf if a == 1 else (cf + cb) if a == 2 else 0) for a in assign)
        if cost > cap:
            continue
        v = sum((so[i] if a == 1 else sf[i] if a == 2 else 0.0) for i, a in enumerate(assign))
        if v > best:
            best, best_assign = v, assign
    assert set(i for i, a in enumerate(best_assign) if a == 2) == full


def test_config3_split_matches_recipe():
    """48 heads, costs (1, 2), budget 60% of all-full: 28 full heads, capacity 2 left for p_o."""
    ks = di.draw_knapsack_inputs(np.random.default_rng(0), 1, 48, 1, 2, 0.6)
    assert int(ks.cap_full[0]) == 86 and int(ks.cap_fwd[0]) == 2
    t = orc.knapsack_scheduling(ks.score_full, ks.score_fwd, ks.cost_fwd, ks.cost_bwd, ks.cap_full, ks.cap_fwd)
    assert (t == FULL).sum() == 28
    assert (t == FULL).sum() * 3 + (t == FWD).sum() <= 88
    top28 = set(np.argsort(-ks.score_full[0])[:28].tolist())
    assert set(np.where(t[0] == FULL)[0].tolist()) == top28


# ---------------------------------------------------------------------------
# analytic cost rules against the values the paper prints
# ---------------------------------------------------------------------------
def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [tuple(float(v) for v in line.split()) for line in f if line.strip() and not line.startswith("#")]


def test_forward_effect_table():
    for n_po, pct in _rows("forward_effect_cost.txt"):
        got = 100.0 * orc.compute_cost_fraction(1, int(n_po), 4 - int(n_po))
        assert abs(got - pct) < 1e-9


def test_comm_cost_rule():
    for n_pf, n_po, n_ps, pct in _rows("comm_cost_rule.txt"):
        got = 100.0 * orc.comm_cost_fraction(int(n_pf), int(n_po), int(n_ps))
        assert abs(got - pct) < 1e-9
