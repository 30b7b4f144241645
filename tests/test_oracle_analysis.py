"""Pins for the oracle's analysis observables: Alg. 1 on given draws (App. H (NormRouter Monte Carlo initialization)) and the
distinct-expert count U(x) (App. E (distinct-expert accounting))."""
import math

import numpy as np
import pytest

from oracle import unipool_oracle as O


def test_c_from_samples_by_loops():
    rng = np.random.default_rng(2)
    E, k, n = 7, 3, 40
    x = rng.standard_normal((n, E))
    x[5] = -np.abs(x[5])                      # a row with no positive component: dropped
    total, used = 0.0, 0
    for r in range(n):
        nrm = math.sqrt(sum(v * v for v in x[r]))
        y = sorted((max(v / nrm, 0.0) for v in x[r]), reverse=True)
        s = math.sqrt(sum(v * v for v in y[:k]))
        if s > 0.0:
            total += 1.0 / s
            used += 1
    c, u = O.c_from_samples(x, k)
    assert u == used == n - 1
    assert c == pytest.approx(total / used, rel=1e-13)


def test_c_from_samples_closed_cases():
    # one expert: y = 1 when x > 0, dropped otherwise -> c = 1
    x = np.array([[0.3], [-1.0], [2.0], [0.01]])
    assert O.c_from_samples(x, 1) == (1.0, 3)
    # k = E and all components positive: the top-k part is the whole unit vector -> 1
    x = np.abs(np.random.default_rng(0).standard_normal((9, 5))) + 0.1
    c, u = O.c_from_samples(x, 5)
    assert u == 9 and c == pytest.approx(1.0, rel=1e-14)
    # scaling a row does not change its term (x / ||x||)
    x2 = x * np.arange(1, 10)[:, None]
    assert O.c_from_samples(x2, 2)[0] == pytest.approx(O.c_from_samples(x, 2)[0], rel=1e-13)
    # a row (3, 4, 0, -1) / sqrt(26) with k = 1 contributes sqrt(26) / 4
    assert O.c_from_samples(np.array([[3.0, 4.0, 0.0, -1.0]]), 1)[0] == pytest.approx(math.sqrt(26.0) / 4.0, rel=1e-14)
    assert O.c_from_samples(np.array([[3.0, 4.0, 0.0, -1.0]]), 2)[0] == pytest.approx(math.sqrt(26.0) / 5.0, rel=1e-14)


def test_distinct_experts_hand_cases():
    # T = 3 tokens, L = 3 layers, k = 2
    l0 = np.array([[0, 1], [2, 3], [4, 5]])
    l1 = np.array([[1, 0], [3, 6], [7, 8]])
    l2 = np.array([[0, 1], [2, 6], [9, 10]])
    U, mean = O.distinct_experts([l0, l1, l2])
    assert U.tolist() == [2, 3, 6] and mean == pytest.approx(11.0 / 3.0)      # {0,1}; {2,3,6}; six different
    # one layer: exactly k
    assert O.distinct_experts([l0])[0].tolist() == [2, 2, 2]


def test_distinct_experts_uniform_routing_closed_form():
    # top-1, every layer picks uniformly and independently: E[U] = M (1 - (1 - 1/M)^L)   (occupancy)
    rng = np.random.default_rng(7)
    M, L, T = 192, 24, 20000
    idx = [rng.integers(0, M, size=(T, 1)) for _ in range(L)]
    U, mean = O.distinct_experts(idx)
    expect = M * (1.0 - (1.0 - 1.0 / M) ** L)
    assert U.min() >= 1 and U.max() <= L
    assert abs(mean - expect) < 0.03          # sd of U is about 1.1; 20000 tokens -> 0.008 per sigma
