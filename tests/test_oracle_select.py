"""Pins for the oracle's expected-accepted-length and verification-length
selection (CPU only): closed forms, the paper's lemmas, brute force."""
import itertools

import numpy as np

from oracle import sv_oracle as O
import svgen


def test_p_gamma_sums_to_one_and_matches_cases():
    rng = np.random.default_rng(0)
    p = rng.random(7)
    for g in range(8):
        pg = O.p_gamma(p, g)
        assert abs(pg.sum() - 1.0) < 1e-14
    # N < gamma: reject at N+1 after N accepts; N = gamma: all accepted
    pg = O.p_gamma(p, 3)
    assert abs(pg[0] - (1 - p[0])) < 1e-15
    assert abs(pg[2] - p[0] * p[1] * (1 - p[2])) < 1e-15
    assert abs(pg[3] - p[0] * p[1] * p[2]) < 1e-15


def test_expectation_equals_sum_of_prefix_products():
    rng = np.random.default_rng(1)
    p = rng.random((5, 9)).astype(np.float32)
    c = O.prefix_products(p)
    assert np.allclose(c, np.cumprod(p.astype(np.float64), axis=1), rtol=1e-15)
    for b in range(5):
        for g in range(10):
            assert abs(O.expected_accepted(p[b], g) - c[b, :g].sum()) < 1e-12


def test_expectation_special_cases():
    assert O.expected_accepted(np.ones(6), 4) == 4.0
    assert O.expected_accepted(np.zeros(6), 4) == 0.0
    q = 0.7
    for g in range(7):
        geo = sum(q ** j for j in range(1, g + 1))
        assert abs(O.expected_accepted(np.full(6, q), g) - geo) < 1e-14


def test_expectation_is_increasing_and_concave():
    # the paper's lemma on E(N | gamma)
    rng = np.random.default_rng(2)
    for _ in range(50):
        p = rng.random(10)
        E = [O.expected_accepted(p, g) for g in range(11)]
        d1 = np.diff(E)
        assert np.all(d1 >= -1e-15)
        assert np.all(np.diff(d1) <= 1e-15)


def test_p_hat_is_sanitised():
    c = O.prefix_products(np.array([[1.5, np.nan, 0.5], [-0.2, 0.5, 0.5]], dtype=np.float32))
    assert np.array_equal(c, np.array([[1.0, 0.0, 0.0], [0.0, 0.0, 0.0]]))


def _brute_best_sum(c, M):
    """max over gamma vectors with sum M of sum_b E_b(gamma_b) (E via prefix sums)."""
    B, k = c.shape
    best = -1.0
    for gam in itertools.product(range(k + 1), repeat=B):
        if sum(gam) == M:
            best = max(best, sum(c[b, :gam[b]].sum() for b in range(B)))
    return best


def test_greedy_set_maximises_expected_length_for_every_budget():
    rng = np.random.default_rng(3)
    for B, k in ((2, 3), (3, 3), (3, 2)):
        for _ in range(10):
            p = rng.random((B, k)).astype(np.float32)
            c = O.prefix_products(p)
            for M in range(1, B * k + 1):
                # a latency table that makes goodput rise up to exactly M tokens
                lat = np.full(B * k + 1, 1.0, dtype=np.float32)
                lat[M + 1:] = 1e9
                gamma, offs, total = O.select_length(p, lat)
                assert total == M and gamma.sum() == M
                got = sum(c[b, :gamma[b]].sum() for b in range(B))
                assert abs(got - _brute_best_sum(c, M)) < 1e-12
                assert np.array_equal(offs, np.concatenate([[0], np.cumsum(gamma + 1)]))


def test_first_peak_is_global_argmax_under_latency_assumption():
    # latency increments non-decreasing (the paper's assumption) => goodput is
    # unimodal and the incremental search finds the global maximum.  Random
    # inputs can produce ties of goodput only with probability zero.
    rng = np.random.default_rng(4)
    for _ in range(200):
        B, k = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        p = rng.random((B, k)).astype(np.float32)
        n = B * k
        m0 = int(rng.integers(1, n + 1))
        lat = svgen.latency_table(n, t0=float(rng.uniform(0.05, 3)), d=float(rng.uniform(0.05, 1)),
                                  m0=m0)
        gamma, _, M = O.select_length(p, lat)
        c = np.sort(O.prefix_products(p).ravel())[::-1]
        good = np.concatenate([[0.0], np.cumsum(c)]) / lat.astype(np.float64)
        assert M == int(np.argmax(good))
        assert np.isclose(good[M], good.max())


def test_single_sequence_equals_incremental_search():
    rng = np.random.default_rng(5)
    for _ in range(100):
        k = int(rng.integers(1, 9))
        p = rng.random((1, k)).astype(np.float32)
        lat = svgen.latency_table(k, t0=float(rng.uniform(0.05, 2)), d=0.3, m0=3)
        # hand-rolled: raise gamma while estimated goodput improves
        g = 0
        good = 0.0
        while g < k:
            nxt = O.expected_accepted(p[0], g + 1) / float(lat[g + 1])
            if nxt > good:
                g, good = g + 1, nxt
            else:
                break
        for mode in (O.MODE_BATCH_GREEDY, O.MODE_PER_SEQUENCE):
            gamma, offs, M = O.select_length(p, lat, mode)
            assert gamma[0] == g and M == g and offs[1] == g + 1


def test_flat_and_steep_latency_and_zero_estimates():
    rng = np.random.default_rng(6)
    p = (0.1 + 0.9 * rng.random((4, 5))).astype(np.float32)
    gamma, _, M = O.select_length(p, np.full(21, 2.0, np.float32))
    assert np.all(gamma == 5) and M == 20
    steep = (10.0 ** np.arange(21)).astype(np.float32)
    gamma, _, M = O.select_length(p, steep)
    assert M == 1 and gamma.sum() == 1
    assert gamma[np.argmax(p[:, 0])] == 1
    gamma, offs, M = O.select_length(np.zeros((3, 4), np.float32), np.ones(13, np.float32))
    assert M == 0 and np.all(gamma == 0) and np.array_equal(offs, [0, 1, 2, 3])


def test_ties_go_to_the_lowest_sequence_then_position():
    p = np.array([[0.5, 1.0], [0.5, 0.4]], dtype=np.float32)   # c = [.5,.5],[.5,.2]
    lat = np.ones(5, np.float32)
    lat[3:] = 1e9
    gamma, _, M = O.select_length(p, lat)
    assert M == 2 and list(gamma) == [2, 0]
    lat = np.ones(5, np.float32)
    lat[4:] = 1e9
    gamma, _, M = O.select_length(p, lat)
    assert M == 3 and list(gamma) == [2, 1]


def test_per_sequence_mode_is_independent_per_sequence():
    rng = np.random.default_rng(7)
    p = rng.random((6, 5)).astype(np.float32)
    lat = svgen.latency_table(5, t0=0.5, d=0.4, m0=2)
    gamma, offs, M = O.select_length(p, lat, O.MODE_PER_SEQUENCE)
    for b in range(6):
        g1, _, _ = O.select_length(p[b:b + 1], lat, O.MODE_PER_SEQUENCE)
        assert gamma[b] == g1[0]
    assert M == gamma.sum() and offs[-1] == M + 6
