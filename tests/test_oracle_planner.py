"""Pins of the oracle's Tier-2 planner (Sec. 6.2 of the paper: workers per ranking group so that the groups' finish
times rise linearly with the smallest gradient the worker budget allows).  The oracle returns the exact optimum; the
paper's bisection approaches it from above to a given precision."""
import itertools

import numpy as np

import oracle


def brute_force(tau, min_wks, wks, t0):
    """Smallest gradient any allocation within the worker budget can meet, by enumeration."""
    n, k = tau.shape
    best = None
    for alloc in itertools.product(range(k), repeat=n):
        if sum(a + min_wks for a in alloc) > wks or tau[0, alloc[0]] > t0:
            continue
        g = max([0.0] + [(tau[i, alloc[i]] - t0) / i for i in range(1, n)])
        best = g if best is None else min(best, g)
    return best


def random_tau(rng, n, k, min_wks):
    lens = np.sort(rng.uniform(200, 16000, n))
    lens[-1] *= rng.uniform(1.0, 4.0)                       # a long-tail group
    ks = np.arange(min_wks, min_wks + k)
    # time ~ length * (serial part + parallel part / workers), roughly what data-parallel rollout workers give
    return lens[:, None] * (0.2 + 0.8 / ks[None, :]) * rng.uniform(0.9, 1.1, (n, 1))


def test_plan_is_feasible_minimal_and_equals_the_brute_force_optimum():
    rng = np.random.default_rng(5)
    seen_none = 0
    for trial in range(300):
        n, k, min_wks = int(rng.integers(2, 5)), int(rng.integers(1, 5)), int(rng.integers(1, 3))
        max_wks = min_wks + k - 1
        tau = random_tau(rng, n, k, min_wks)
        wks = int(rng.integers(n * min_wks, n * max_wks + 2))
        t_train = float(rng.choice([0.0, rng.uniform(0, tau[0, 0] * 1.5)]))
        t0 = max(tau[0, -1], t_train)
        got = oracle.plan_allocation(tau, min_wks, max_wks, wks, t_train)
        d_top = max(0.0, (tau[-1, 0] - t0) / (n - 1))
        best = brute_force(tau, min_wks, wks, t0)
        if got is None:
            # nothing in the search interval [0, d_top] is affordable (at d_top itself the last group's target,
            # t0 + (n-1) d_top, can fall one rounding short of its time on MIN_WKS workers)
            assert best is None or best >= d_top * (1 - 1e-12)
            seen_none += 1
            continue
        plan, d = got
        assert plan.sum() <= wks and plan.min() >= min_wks and plan.max() <= max_wks
        for i in range(n):
            assert tau[i, plan[i] - min_wks] <= t0 + i * d                       # meets its target time
            if plan[i] > min_wks:
                assert tau[i, plan[i] - 1 - min_wks] > t0 + i * d               # with the fewest workers
        # the enumeration's optimum, exactly (up to the rounding of (tau - t0) / i)
        assert best is not None and abs(d - max(best, 0.0)) <= 1e-9 * (1.0 + abs(best)), (trial, d, best)
    assert 10 < seen_none < 200


def test_reshaping_gives_long_groups_more_workers():
    # eight groups whose lengths grow exponentially (the long tail of Sec. 6.2); time = length / workers
    lens = 500.0 * 1.6 ** np.arange(8)
    min_wks, max_wks = 1, 8
    tau = lens[:, None] / np.arange(min_wks, max_wks + 1)[None, :]
    # the training stage takes longer than the shortest group on one worker: t0 = t_train
    plan, d = oracle.plan_allocation(tau, min_wks, max_wks, wks=24, t_train=600.0)
    assert plan.sum() <= 24 and plan[0] == 1 and plan[-1] == plan.max() > 3
    finish = lens / plan
    even = lens / 3.0                                           # the same 24 workers spread evenly
    assert finish.max() < even.max()
    # finish times stay under the line t0 + i d
    assert np.all(finish <= 600.0 + np.arange(8) * d + 1e-9)
    # with t_train = 0 the figure's t0 = tau(lens[0], MAX_WKS) asks the shortest group for its fastest time
    plan0, _ = oracle.plan_allocation(tau, min_wks, max_wks, wks=24, t_train=0.0)
    assert plan0[0] == max_wks
    # more workers never make the gradient worse
    d_prev = None
    for wks in range(10, 60, 5):
        r = oracle.plan_allocation(tau, min_wks, max_wks, wks, 0.0)
        if r is not None:
            assert d_prev is None or r[1] <= d_prev + 1e-12
            d_prev = r[1]


def test_training_time_sets_the_floor_and_single_group():
    tau = np.array([[40.0, 25.0, 18.0], [90.0, 50.0, 35.0]])
    plan, d = oracle.plan_allocation(tau, 1, 3, wks=6, t_train=60.0)
    assert plan[0] == 1                                  # t0 = 60: the first group already meets it on one worker
    plan2, d2 = oracle.plan_allocation(tau, 1, 3, wks=6, t_train=0.0)
    assert plan2[0] == 3 and plan2.tolist() == [3, 3]    # t0 = tau(lens[0], MAX_WKS) = 18: group 1 needs 35 <= 18 + d
    assert abs(d2 - 17.0) < 1e-9
    one = oracle.plan_allocation(tau[:1], 1, 3, wks=3, t_train=30.0)
    assert one[0].tolist() == [2] and one[1] == 0.0
    assert oracle.plan_allocation(tau, 1, 3, wks=1, t_train=0.0) is None
