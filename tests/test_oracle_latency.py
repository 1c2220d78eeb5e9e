"""Pins for the oracle's run-time model (Section III-C, eq. (5), Appendix D, Theorem 2)."""
import math

import numpy as np
import pytest

from oracle import cr_tree, latency


def test_inverse_cdf_of_eq_5():
    a, mu, d = 5e-5, 2e4, 8320
    for t in [a * d, a * d + 0.1, a * d + 1.0, a * d + 3.0]:
        u = 1.0 - math.exp(-(mu / d) * (t - a * d))      # eq. (5)
        assert latency.compute_time(u, d, a, mu) == pytest.approx(t, rel=1e-12, abs=1e-12)
    assert latency.compute_time(0.0, d, a, mu) == a * d  # the shift is the minimum


def test_worked_single_port_example():
    # one layer, 3 children, 1 straggler; exponential parts 0, 1, 2 time units; t_c = 0.3
    a, mu, d, t_c = 0.01, 50.0, 100, 0.3                  # shift = 1.0, scale d/mu = 2.0
    u = [0.0, 1 - math.exp(-0.5), 1 - math.exp(-1.0)]     # T = 1.0, 2.0, 3.0
    mask, ready, total = latency.simulate_iteration(1, 3, 1, [d] * 3, a, mu, t_c, u)
    assert ready == pytest.approx([1.0, 2.0, 3.0])
    assert mask == [0, 0, 1]
    assert total == pytest.approx(2.3)                    # child 0 received at 1.3, child 1 sends 2.0 -> 2.3
    # a busy port delays the second transfer
    mask, ready, total = latency.simulate_iteration(1, 3, 1, [d] * 3, a, mu, 1.5, u)
    assert total == pytest.approx(1.0 + 1.5 + 1.5) and mask == [0, 0, 1]
    # the slowest child is dropped whichever index it has
    mask, _, _ = latency.simulate_iteration(1, 3, 1, [d] * 3, a, mu, t_c, [u[2], u[0], u[1]])
    assert mask == [1, 0, 0]


def test_two_layers_by_hand():
    # (2,2) tree, s = 1: every parent waits for its faster child only
    a, mu, t_c = 0.0, 1.0, 0.25
    rows = [1] * 6
    E = [0.5, 4.0, 1.0, 3.0, 0.2, 0.3]                    # exponential parts = compute times (a = 0, rows/mu = 1)
    u = [1 - math.exp(-e) for e in E]
    mask, ready, total = latency.simulate_iteration(2, 2, 1, rows, a, mu, t_c, u)
    assert ready[2:] == pytest.approx([1.0, 3.0, 0.2, 0.3])
    assert ready[0] == pytest.approx(max(0.5, 1.0 + 0.25))          # node (1,1): faster child (2,1) at 1.0
    assert ready[1] == pytest.approx(max(4.0, 0.2 + 0.25))          # node (1,2): own computation is the slow part
    assert total == pytest.approx(1.25 + 0.25)
    assert mask == [0, 1, 0, 1, 0, 1]


def test_mean_order_statistic_closed_form():
    # Appendix D: E[T_(n-s)] = (rows/mu)(H_n - H_s) + a rows; one layer, free communication
    n, s, rows, a, mu = 12, 3, 500, 1e-3, 100.0
    totals = [latency.simulate(1, n, s, [rows] * n, a, mu, 0.0, seed=7, iteration=t)[2] for t in range(20000)]
    expect = latency.expected_order_statistic(n, s, rows, a, mu)
    assert expect == pytest.approx((rows / mu) * sum(1.0 / i for i in range(s + 1, n + 1)) + a * rows)
    assert np.mean(totals) == pytest.approx(expect, rel=0.01)


@pytest.mark.parametrize("L,n,s", [(1, 6, 2), (2, 4, 1), (3, 3, 1), (2, 12, 5)])
def test_structure_and_hard_bounds(L, n, s):
    N = cr_tree.num_workers(n, L)
    rng = np.random.default_rng(L * 100 + n)
    rows = [int(v) for v in rng.integers(50, 60, size=N)]
    a, mu, t_c = 2e-3, 40.0, 0.07
    for it in range(50):
        mask, ready, total = latency.simulate(L, n, s, rows, a, mu, t_c, seed=3, iteration=it)
        T = [latency.compute_time(latency.uniform01(3, it * N + k), rows[k], a, mu) for k in range(N)]
        for g in range(N // n):                          # exactly s stragglers per group: the s last to become ready
            grp = list(range(g * n, (g + 1) * n))
            assert sum(mask[k] for k in grp) == s
            slow = sorted(grp, key=lambda k: (ready[k], k))[n - s:]
            assert sorted(k for k in grp if mask[k]) == sorted(slow)
        assert all(ready[k] >= T[k] for k in range(N))
        assert total >= min(a * r for r in rows) + (n - s + L - 1) * t_c - 1e-12
        assert total <= max(T) + L * (n - s) * t_c + 1e-12


def test_saturated_port_and_theorem_2_shape():
    # communication-dominated regime (t_c larger than the gaps between arrivals): a group costs first arrival + (n-s) t_c
    n, s, rows, a, mu, t_c = 16, 4, 100, 1e-3, 1000.0, 5.0
    for it in range(20):
        _, ready, total = latency.simulate(1, n, s, [rows] * n, a, mu, t_c, seed=11, iteration=it)
        assert total == pytest.approx(min(ready) + (n - s) * t_c)
    # Theorem 2 with its o(.) terms dropped: compute term + between (n(1-alpha) + L - 1) t_c and n L t_c
    L, n, s = 2, 48, 12
    N = cr_tree.num_workers(n, L)
    r = float(cr_tree.computation_load(n, L, s))
    m = 10 ** 6
    rows = [r * m] * N
    a, mu, t_c = 1e-6, 1e5, 0.05
    totals = [latency.simulate(L, n, s, rows, a, mu, t_c, seed=5, iteration=t)[2] for t in range(200)]
    compute = (r * m / mu) * math.log(n / s) + a * r * m
    assert compute + (n - s + L - 1) * t_c * 0.95 <= np.mean(totals) <= compute * 1.3 + n * L * t_c
