"""The C++ dispatcher (through its C ABI) against the exhaustive oracle, plus host-side checks.
Host code only: these run without a GPU."""
import os
import re
import time

import numpy as np
import pytest

from oracle import dispatch_oracle as DO

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def T():
    from paper_2510_02838_amd import dispatch
    return dispatch


def test_library_exports_every_declared_dispatch_symbol(T):
    hdr = open(os.path.join(ROOT, "include", "dispatch.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(tds_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(T.EXPORTS) and len(declared) == 3


def _instance(rng, R, I=4, K=4, p_feas=0.5, tight=True):
    t1 = rng.uniform(0.5, 20.0, (R, I, 1))
    speed = np.array([1.0, 1.9, 3.5, 6.0])[:K]
    t = t1 / speed
    feas = (rng.random((R, I, K)) < p_feas).astype(np.uint8)
    deadline = rng.uniform(1.0, 15.0, R)
    length = rng.uniform(64, 60000, R)
    B = rng.integers(0, 6 if tight else 40, I)
    return t, feas, deadline, length, B


def _check_valid(choice, feas, B, degrees):
    used = [0] * feas.shape[1]
    for r, c in enumerate(choice):
        if c is None:
            continue
        i, k = c
        assert feas[r, i, degrees.index(k)], (r, c)
        used[i] += k
    assert all(u <= b for u, b in zip(used, B)), (used, B)


def test_weights_and_penalties_equal_the_oracles(T):
    rng = np.random.default_rng(1)
    for _ in range(20):
        t, feas, deadline, length, B = _instance(rng, 9)
        tau = float(rng.uniform(0, 3))
        assert np.array_equal(T.reward_weights(t, feas, deadline, tau), DO.reward_weights(t, feas, deadline, tau))
        assert np.array_equal(T.comm_penalty(length), DO.comm_penalty(length))
    # a lower starvation threshold can only raise the reward of late requests
    assert (T.reward_weights(t, feas, deadline, tau, alpha=2.0) >= T.reward_weights(t, feas, deadline, tau)).all()


@pytest.mark.parametrize("seed", range(40))
def test_solver_equals_exhaustive_search(T, seed):
    rng = np.random.default_rng(100 + seed)
    R = int(rng.integers(1, 6))
    I = int(rng.integers(1, 5))
    t, feas, deadline, length, B = _instance(rng, R, I=I, p_feas=float(rng.uniform(0.2, 0.9)), tight=True)
    tau = float(rng.uniform(0, 2))
    W = DO.reward_weights(t, feas, deadline, tau)
    Q = DO.comm_penalty(length)[:, :I]
    want, _ = DO.solve_bruteforce(W, Q, feas, list(B))
    got = T.solve(W, Q, feas, B, t, deadline, tau)
    assert got["status"] == T.TDS_OK
    _check_valid(got["choice"], feas, list(B), list(DO.DEGREES))
    assert got["objective"] == pytest.approx(DO.objective(got["choice"], W, Q), rel=1e-12, abs=1e-12)
    assert got["objective"] == pytest.approx(want, rel=1e-12, abs=1e-9)
    assert got["upper_bound"] == pytest.approx(got["objective"], abs=1e-9)
    assert got["D"] == DO.on_time(got["choice"], t, deadline, tau)


def test_equal_values_with_reward_ties_and_odd_capacity(T):
    # 60 identical on-time requests that need 8 replicas each, 100 idle: 12 fit; without the
    # capacity rounding in the bound this enumerates subsets
    R = 60
    feas = np.zeros((R, 1, 4), np.uint8); feas[:, 0, 3] = 1
    t = np.ones((R, 1, 4)); deadline = np.full(R, 10.0)
    W = np.full(R, 1000.0); Q = np.zeros((R, 1))
    got = T.solve(W, Q, feas, [100], t, deadline, 0.0, node_limit=200000)
    assert got["status"] == T.TDS_OK and got["objective"] == 12000.0 and got["nodes"] < 5000
    assert sum(got["D"]) == 12


def test_prefers_less_communication_among_equal_rewards(T):
    # two on-time requests, one <EDC> replica and one <D> replica: the longer request gets <EDC>
    feas = np.zeros((2, 4, 4), np.uint8); feas[:, 0, 0] = 1; feas[:, 3, 0] = 1
    t = np.ones((2, 4, 4)); deadline = [5.0, 5.0]
    W = DO.reward_weights(t, feas, deadline, 0.0)
    Q = DO.comm_penalty([1000.0, 50000.0])
    got = T.solve(W, Q, feas, [1, 0, 0, 1], t, deadline, 0.0)
    assert got["choice"] == [(3, 1), (0, 1)]
    assert got["objective"] == pytest.approx(2000.0 - 6e-6 * 1000.0)


def test_on_time_requests_win_over_late_ones(T):
    # capacity for one of two: the on-time request (1000) beats the late one (200)
    feas = np.zeros((2, 1, 4), np.uint8); feas[:, 0, 0] = 1
    t = np.array([[[9.0] * 4], [[2.0] * 4]]); deadline = [3.0, 3.0]
    W = DO.reward_weights(t, feas, deadline, 0.0)
    got = T.solve(W, np.zeros((2, 1)), feas, [1], t, deadline, 0.0)
    assert got["choice"] == [None, (0, 1)] and got["D"] == [0, 1]


def test_invalid_arguments_are_rejected(T):
    feas = np.ones((2, 1, 4), np.uint8); t = np.ones((2, 1, 4))
    with pytest.raises(ValueError):
        T.solve([1.0, np.nan], np.zeros((2, 1)), feas, [1], t, [1.0, 1.0], 0.0)
    with pytest.raises(ValueError):
        T.solve([1.0, 1.0], np.zeros((2, 1)), feas, [-1], t, [1.0, 1.0], 0.0)
    with pytest.raises(ValueError):
        T.solve([1.0, 1.0], np.zeros((2, 1)), feas, [1], t, [1.0, 1.0], 0.0, degrees=(1, 2, 2, 8))
    with pytest.raises(ValueError):
        T.solve([1.0] * 2, np.zeros((2, 5)), np.ones((2, 5, 4), np.uint8), [1] * 5, np.ones((2, 5, 4)), [1.0] * 2, 0.0)


def test_node_limit_returns_a_valid_assignment_and_a_bound(T):
    rng = np.random.default_rng(5)
    t, feas, deadline, length, B = _instance(rng, 300, tight=False)
    W = DO.reward_weights(t, feas, deadline, 0.0); Q = DO.comm_penalty(length)
    got = T.solve(W, Q, feas, B, t, deadline, 0.0, node_limit=50)
    assert got["status"] == T.TDS_LIMIT
    _check_valid(got["choice"], feas, list(B), list(DO.DEGREES))
    assert got["upper_bound"] >= got["objective"] - 1e-9


@pytest.mark.parametrize("gpus", [128, 1024, 4096])
def test_cluster_scale_tick_solves_fast_and_tight(T, gpus):
    """A scheduling tick at the cluster sizes of the paper's dispatcher-scalability table
    (128 to 4096 GPUs): queue of gpus/4 requests, a quarter of the GPUs idle, two Primary types.
    Within its node budget the search must return an assignment proven to be within one
    on-time reward (1000) of the optimum, out of an objective of 3e4 to 1e6."""
    rng = np.random.default_rng(gpus)
    R = gpus // 4
    t, feas, deadline, length, _ = _instance(rng, R, p_feas=0.7)
    feas[:, 1:3] = 0                                   # types <EDC> and <D> only
    B = [gpus // 8, 0, 0, gpus // 8]
    W = DO.reward_weights(t, feas, deadline, 0.0); Q = DO.comm_penalty(length)
    t0 = time.perf_counter()
    got = T.solve(W, Q, feas, B, t, deadline, 0.0, node_limit=300_000, gap_abs=1e-3)
    dt = time.perf_counter() - t0
    _check_valid(got["choice"], feas, B, list(DO.DEGREES))
    assert got["upper_bound"] - got["objective"] < 1000.0
    assert dt < 5.0
