"""Pins of the dispatcher oracle against what the paper prints and what the mathematics fixes."""
import os

import numpy as np
import pytest

from oracle import dispatch_oracle as DO

HERE = os.path.dirname(os.path.abspath(__file__))


def test_constants_are_the_papers():
    # Appendix "Dispatch Plan", paragraph "Constant values"
    assert (DO.C_ON, DO.C_LATE, DO.ALPHA) == (1000.0, 200.0, 5.0)
    assert DO.BETA == (0.0, 1e-6, 5e-6, 6e-6)
    assert DO.DEGREES == (1, 2, 4, 8)                       # set K of the integer program


def test_reward_matches_the_papers_worked_examples():
    rows = [l.split() for l in open(os.path.join(HERE, "golden", "dispatch_reward_examples.txt")) if l[0] != "#"]
    assert len(rows) == 3
    for alpha, scale, mult in rows:
        alpha, scale, mult = float(alpha), float(scale), float(mult)
        # one request, one option, deadline 1, tau 0, runtime = scale  =>  T_hat / d = scale
        W = DO.reward_weights([[[scale]]], [[[1]]], [1.0], 0.0, alpha=alpha)
        assert W[0] == pytest.approx(mult * DO.C_LATE, rel=1e-12)


def test_reward_on_time_late_boundary_and_tau():
    t = np.array([[[3.0, 2.0]], [[3.0, 2.0]], [[3.0, 2.0]], [[30.0, 20.0]]])
    feas = np.ones_like(t)
    # tau = 1: best completion 3.0; deadlines 3.0 (equal: on time), 2.99 (late, scale ~1), 10, and 3 (scale 7)
    W = DO.reward_weights(t, feas, [3.0, 2.99, 10.0, 3.0], 1.0)
    assert W[0] == 1000.0 and W[2] == 1000.0
    assert W[1] == 200.0
    assert W[3] == pytest.approx(200.0 * (21.0 / 3.0 - 5.0 + 1.0))       # scale 7 -> 3 * C_late


def test_reward_uses_only_feasible_options():
    t = np.array([[[1.0, 9.0], [2.0, 9.0]]])          # the fast options are filtered out
    feas = np.array([[[0, 1], [0, 1]]])
    assert DO.reward_weights(t, feas, [5.0], 0.0)[0] == 200.0     # T_hat = 9 > 5: late, scale 1.8
    feas[0, 1, 0] = 1
    assert DO.reward_weights(t, feas, [5.0], 0.0)[0] == 1000.0    # T_hat = 2
    assert DO.reward_weights(t, np.zeros_like(feas), [5.0], 0.0)[0] == 0.0


def test_penalty_is_linear_ordered_and_small():
    Q = DO.comm_penalty([1000.0, 4096.0, 1e6])
    assert Q.shape == (3, 4)
    assert np.all(Q[:, 0] == 0.0)
    assert Q[1, 1] == pytest.approx(4096e-6) and Q[1, 2] == pytest.approx(5 * 4096e-6) and Q[1, 3] == pytest.approx(6 * 4096e-6)
    assert np.all(np.diff(Q, axis=1) >= 0)            # <EDC> cheapest ... <D> dearest
    assert Q.max() < DO.C_LATE / 10                   # orders of magnitude below any reward


def _knapsack_dp(values, weights, cap):
    best = [0.0] * (cap + 1)
    for v, w in zip(values, weights):
        for c in range(cap, w - 1, -1):
            best[c] = max(best[c], best[c - w] + v)
    return best[cap]


def test_bruteforce_closed_forms():
    rng = np.random.default_rng(7)
    R = 5
    W = rng.choice([1000.0, 200.0, 400.0], R)
    Q = DO.comm_penalty(rng.uniform(100, 5000, R))
    feas = (rng.random((R, 4, 4)) < 0.5).astype(int)
    feas[0] = 0                                        # one request with nothing feasible
    # ample capacity: every dispatchable request goes to its cheapest feasible type
    best, arg = DO.solve_bruteforce(W, Q, feas, [100] * 4)
    want = sum(W[r] - min(Q[r][i] for i in range(4) if feas[r, i].any()) for r in range(R) if feas[r].any())
    assert best == pytest.approx(want, rel=1e-12)
    assert arg[0] is None
    # no capacity: nothing dispatched
    best, arg = DO.solve_bruteforce(W, Q, feas, [0] * 4)
    assert best == 0.0 and all(c is None for c in arg)


def test_bruteforce_single_type_is_the_textbook_knapsack():
    rng = np.random.default_rng(11)
    for trial in range(6):
        R = 6
        W = rng.choice([1000.0, 200.0, 600.0, 800.0], R)
        Q = np.zeros((R, 4))
        feas = np.zeros((R, 4, 4), int)
        ks = rng.integers(0, 4, R)                     # each request has exactly one degree on type 2
        for r in range(R):
            feas[r, 2, ks[r]] = 1
        cap = int(rng.integers(1, 14))
        best, arg = DO.solve_bruteforce(W, Q, feas, [0, 0, cap, 0])
        weights = [DO.DEGREES[k] for k in ks]
        assert best == pytest.approx(_knapsack_dp(list(W), weights, cap))
        assert sum(c[1] for c in arg if c is not None) <= cap       # degree k uses k replicas (C2)


def test_on_time_indicator():
    t = np.array([[[1.0, 0.6, 0.4, 0.3]] * 4, [[5.0, 3.0, 2.0, 1.5]] * 4])
    D = DO.on_time([(0, 1), (3, 4)], t, [1.0, 1.9], 0.0)
    assert D == [1, 0]
    assert DO.on_time([None, (3, 8)], t, [1.0, 1.9], 0.0) == [0, 1]
    assert DO.on_time([(0, 1), (3, 8)], t, [1.0, 1.9], 0.5) == [0, 0]
