"""Pins for the oracle's routing statistics (Sec. Locality Loss) and capacity lower bound
(Remark of Sec. Dynamic Lower Bound Module): CPU only."""
import math

import numpy as np
import pytest
from scipy import stats as sps
from scipy.special import softmax

TCR, ECR, BIDIR = 0, 1, 2


def test_route_stats_against_library_and_brute_force(oracle):
    rng = np.random.default_rng(0)
    T, E, k, C = 500, 7, 2, 90
    S = rng.uniform(-1, 1, (T, E)).astype(np.float32)
    gate = softmax(S.astype(np.float64), axis=1).astype(np.float32)
    _, slot_of, _, counts = oracle.select(S, k, C, TCR)
    target = rng.uniform(0.1, 1.0, E)
    target = (target / target.sum()).astype(np.float32)
    load, mg, kl, un = oracle.route_stats(gate, slot_of, counts, target)
    np.testing.assert_allclose(load, counts / counts.sum(), rtol=1e-15)
    np.testing.assert_allclose(load.sum(), 1.0, rtol=1e-14)
    np.testing.assert_allclose(mg, gate.astype(np.float64).mean(0), rtol=1e-12)
    np.testing.assert_allclose(mg.sum(), 1.0, rtol=1e-6)                 # softmax rows sum to one
    np.testing.assert_allclose(kl, sps.entropy(load, target.astype(np.float64)), rtol=1e-6)    # library KL (it renormalises the fp32 target)
    np.testing.assert_allclose(kl, float(np.sum(load * np.log(load / target.astype(np.float64)))), rtol=1e-13)
    assert kl >= 0                                                        # Gibbs' inequality
    assert un == int(((slot_of >= 0).sum(1) == 0).sum()) and un > 0


def test_kl_special_cases(oracle):
    E, T = 4, 8
    gate = np.full((T, E), 0.25, np.float32)
    slot_of = np.full((T, E), -1, np.int32)
    uniform = np.full(E, 0.25, np.float32)
    # identical distributions: zero
    _, _, kl, un = oracle.route_stats(gate, slot_of, np.array([3, 3, 3, 3]), uniform)
    assert kl == 0.0 and un == T
    # two experts, closed form: D_c = (3/4, 1/4, 0, 0) against uniform
    load, _, kl, _ = oracle.route_stats(gate, slot_of, np.array([6, 2, 0, 0]), uniform)
    np.testing.assert_allclose(kl, 0.75 * math.log(3) + 0.25 * math.log(1), rtol=1e-14)
    assert load.tolist() == [0.75, 0.25, 0, 0]
    # mass where the localized distribution has none: infinite; no mass there: finite
    _, _, kl, _ = oracle.route_stats(gate, slot_of, np.array([6, 2, 0, 0]), np.array([0.5, 0, 0.25, 0.25], np.float32))
    assert math.isinf(kl)
    _, _, kl, _ = oracle.route_stats(gate, slot_of, np.array([6, 2, 0, 0]), np.array([0.5, 0.5, 0, 0], np.float32))
    np.testing.assert_allclose(kl, 0.75 * math.log(1.5) + 0.25 * math.log(0.5), rtol=1e-14)
    # nothing kept at all: all-zero load, zero divergence
    load, _, kl, _ = oracle.route_stats(gate, slot_of, np.array([0, 0, 0, 0]), uniform)
    assert kl == 0.0 and not load.any()
    # asymmetry guard (KL(D_c || D_l), not the reverse)
    _, _, a, _ = oracle.route_stats(gate, slot_of, np.array([9, 1, 0, 0]), np.array([0.5, 0.5, 0, 0], np.float32))
    np.testing.assert_allclose(a, sps.entropy([0.9, 0.1], [0.5, 0.5]), rtol=1e-7)
    assert abs(a - sps.entropy([0.5, 0.5], [0.9, 0.1])) > 0.1


@pytest.mark.parametrize("d,n,dmax,T,expect", [
    (2, 1, 1.0, 100, 8),        # exp(2*1/(2-1)) = e^2 = 7.39 -> 8
    (2, 4, 1.0, 100, 2),        # e^2 / 4 = 1.85 -> 2
    (64, 8, 0.0, 100, 1),       # exp(0)/8 = 0.125 -> ceil 1
    (64, 8, 0.25, 1000, 1),     # exp(64*0.0625/1.9375)/8 = exp(2.0645)/8 = 0.985 -> 1
    (64, 8, 0.5, 2000, 1169),   # exp(64*0.25/1.75)/8 = exp(9.142857)/8 = 1168.43 -> 1169
    (4096, 16, 0.3, 8192, 8192),  # astronomically large: clamped to T
    (10, 2, -0.5, 50, 3),       # only dmax^2 enters: exp(10*0.25/1.75)/2 = 2.086 -> 3
])
def test_capacity_lower_bound_closed_form(oracle, d, n, dmax, T, expect):
    rng = np.random.default_rng(1)
    S = rng.uniform(-1, 1, (T, n)).astype(np.float32)
    S = np.minimum(S, np.float32(dmax) - np.float32(0.01)).astype(np.float32)   # everything below the planted maximum
    S[T // 3, n // 2] = dmax
    dm, c = oracle.capacity_lower_bound(S, d)
    assert dm == np.float32(dmax)
    cmin = math.exp(d * float(np.float32(dmax)) ** 2 / (2 - float(np.float32(dmax)) ** 2)) / n if d < 1000 else float("inf")
    assert c == expect == max(1, min(T, math.ceil(cmin) if math.isfinite(cmin) else T))


def test_capacity_lower_bound_is_monotone(oracle):
    T, n, d = 4096, 8, 64
    prev = 0
    for dmax in np.linspace(0.0, 0.9, 19):
        S = np.full((T, n), -1.0, np.float32)
        S[5, 3] = dmax
        _, c = oracle.capacity_lower_bound(S, d)
        assert 1 <= c <= T and c >= prev
        prev = c
    assert prev == T
