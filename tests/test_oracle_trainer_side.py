"""Pins for oracle/trainer_side.py: the decoupled PPO objective (Eq. 5) against
its own first form, against the standard clipped objective when the proximal
policy is the behaviour policy, and on hand-worked clipping cases; Algorithm 1
(dynamic batching) on a hand-worked example and by its invariants."""
import math

import numpy as np

from oracle import trainer_side as ts


def test_two_forms_of_the_decoupled_objective_agree():
    """Eq. 5, first line: min((pi_theta/pi_behav) A, (pi_prox/pi_behav) clip(pi_theta/pi_prox) A)."""
    rng = np.random.default_rng(0)
    lt, lp, lb = (rng.normal(-3, 1, 500) for _ in range(3))
    a = rng.normal(0, 1, 500)
    eps = 0.2
    total, obj, _ = ts.decoupled_ppo_objective(lt, lp, lb, a, eps)
    first = np.minimum(np.exp(lt - lb) * a,
                       np.exp(lp - lb) * np.clip(np.exp(lt - lp), 1 - eps, 1 + eps) * a)
    np.testing.assert_allclose(obj, first, rtol=1e-12, atol=1e-12)
    assert abs(total - first.sum()) < 1e-9


def test_prox_equal_behav_is_the_standard_clipped_objective():
    rng = np.random.default_rng(1)
    lt, lold = rng.normal(-2, 0.5, 200), rng.normal(-2, 0.5, 200)
    a = rng.normal(0, 1, 200)
    _, obj, _ = ts.decoupled_ppo_objective(lt, lold, lold, a, 0.2)
    u = np.exp(lt - lold)
    std = np.array([min(x * y, min(max(x, 0.8), 1.2) * y) for x, y in zip(u, a)])
    np.testing.assert_allclose(obj, std, rtol=1e-12)


def test_clipping_cases_by_hand():
    ln = math.log
    # (pi_theta, pi_prox, pi_behav, A) -> objective with eps = 0.2
    cases = [((0.6, 0.4, 0.5, 2.0), (0.4 / 0.5) * 1.2 * 2.0),      # u = 1.5 > 1.2, A > 0: clipped
             ((0.2, 0.4, 0.5, 2.0), (0.4 / 0.5) * 0.5 * 2.0),      # u = 0.5, A > 0: min takes the unclipped term
             ((0.2, 0.4, 0.5, -1.0), (0.4 / 0.5) * 0.8 * -1.0),    # u = 0.5 < 0.8, A < 0: clipped
             ((0.6, 0.4, 0.5, -1.0), (0.4 / 0.5) * 1.5 * -1.0),    # u = 1.5, A < 0: unclipped (more negative)
             ((0.4, 0.4, 0.1, 3.0), 4.0 * 3.0)]                    # theta = prox: weight pi_prox/pi_behav only
    for (pt, pp, pb, adv), want in cases:
        total, _, _ = ts.decoupled_ppo_objective([ln(pt)], [ln(pp)], [ln(pb)], [adv], 0.2)
        assert abs(total - want) < 1e-12
    total, obj, clipped = ts.decoupled_ppo_objective([ln(0.6), ln(0.2)], [ln(0.4)] * 2, [ln(0.5)] * 2, [2.0, 2.0],
                                                    0.2, mask=[True, False])
    assert abs(total - 1.92) < 1e-12 and obj[1] == 0.0 and clipped.tolist() == [True, False]


def test_dynamic_batching_worked_example():
    # lengths sorted: 9 8 7 4 3 2 1; C = 10, k_min = 2
    # 9 -> new (fewer than 2 batches); 8 -> new; 7 -> no room anywhere -> new;
    # 4 -> fits nowhere (9+4, 8+4, 7+4 > 10) -> new; 3 -> fits {7}(10) and {4}(7): one sequence each,
    # earlier wins -> {7,3}; 2 -> fits {8}(10), {4}(6): {8,2}; 1 -> fits {9}(10), {4}(5): {9,1}
    lens = [3, 9, 1, 7, 2, 8, 4]
    got = ts.dynamic_batching(lens, 10, 2)
    assert [[lens[i] for i in b] for b in got] == [[9, 1], [8, 2], [7, 3], [4]]


def test_dynamic_batching_invariants():
    rng = np.random.default_rng(2)
    for _ in range(50):
        n = int(rng.integers(1, 40))
        lens = rng.integers(1, 50, size=n)
        cap = int(rng.integers(20, 120))
        k = int(rng.integers(1, 6))
        got = ts.dynamic_batching(lens, cap, k)
        flat = sorted(i for b in got for i in b)
        assert flat == list(range(n))                                    # a partition
        for b in got:
            assert sum(lens[i] for i in b) <= cap or len(b) == 1         # capacity (oversize: alone)
        assert len(got) >= min(k, n)                                     # at least k_min micro-batches
    assert ts.dynamic_batching([], 10, 3) == []
    assert ts.dynamic_batching([50], 10, 1) == [[0]]
