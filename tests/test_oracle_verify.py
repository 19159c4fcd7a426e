"""Pins for the oracle's speculative-sampling verification (CPU only).

The law of the emitted tokens is fixed by mathematics, not by any
implementation: every emitted token follows the target distribution given its
prefix, whichever prefix of the draft is verified.  The checks below derive
that law from toy model tables and compare it with what the oracle emits."""
import itertools

import numpy as np
import scipy.special

from oracle import philox
from oracle import sv_oracle as O


def _softmax(z):
    return scipy.special.softmax(np.asarray(z, dtype=np.float64), axis=-1)


def test_acceptance_probability_is_one_minus_tv():
    rng = np.random.default_rng(0)
    for V in (2, 5, 8, 64):
        zt = rng.standard_normal(V) * 2
        zd = zt + rng.standard_normal(V)
        pt, pd = _softmax(zt), _softmax(zd)
        acc = sum(pd[t] * min(1.0, O.accept_ratio(zt, zd, t)[0]) for t in range(V))
        assert abs(acc - np.minimum(pt, pd).sum()) < 1e-13
        assert abs(acc - (1 - 0.5 * np.abs(pt - pd).sum())) < 1e-13
        for t in range(V):
            assert abs(O.accept_ratio(zt, zd, t)[0] - pt[t] / pd[t]) < 1e-12 * pt[t] / pd[t]


def test_one_position_emits_the_target_distribution():
    # sum_x P_d(x) [ a(x) 1{x = y} + (1 - a(x)) r(y) ] = P_t(y)
    rng = np.random.default_rng(1)
    for V in (2, 3, 8):
        for _ in range(20):
            zt = rng.standard_normal(V) * 2
            zd = rng.standard_normal(V) * 2
            pt, pd = _softmax(zt), _softmax(zd)
            w, W, fl = O.sampling_weights(zt, zd)
            assert fl == 0
            emitted = np.zeros(V)
            for t in range(V):
                a = min(1.0, O.accept_ratio(zt, zd, t)[0])
                emitted[t] += pd[t] * a
                emitted += pd[t] * (1 - a) * w / W
            assert np.allclose(emitted, pt, atol=1e-13)


def test_inverse_cdf_matches_searchsorted_and_interval_measures():
    rng = np.random.default_rng(2)
    w = rng.random(9)
    w[[2, 5]] = 0.0
    W = float(np.cumsum(w)[-1])
    J = 20000
    counts = np.zeros(9)
    for j in range(J):
        u = (j + 0.5) / J
        y, margin, adm = O.inverse_cdf(w, W, u)
        assert y == int(np.searchsorted(np.cumsum(w), u * W, side="right"))
        assert y in adm and margin >= 0
        counts[y] += 1
    assert np.allclose(counts / J, w / W, atol=1.5 / J)
    assert counts[2] == 0 and counts[5] == 0


def test_inverse_cdf_edges_and_fallback():
    w = np.array([0.25, 0.0, 0.5, 0.25, 0.0])
    # threshold exactly on an edge belongs to the next positive token
    y, margin, adm = O.inverse_cdf(w, 1.0, 0.25)
    assert y == 2 and margin == 0.0 and set(adm) == {0, 2}
    # rounding: threshold at/above the total -> last positive-weight token
    y, _, _ = O.inverse_cdf(w, 1.0 + 1e-12, 1.0)
    assert y == 3
    y, margin, adm = O.inverse_cdf(w, 1.0, 0.5)
    assert y == 2 and abs(margin - 0.25) < 1e-15 and list(adm) == [2]


def _toy_tables(rng, V, depth, temp=1.5):
    """Context-dependent toy models: one logit row per prefix of length < depth."""
    tab = {}
    for L in range(depth):
        for prefix in itertools.product(range(V), repeat=L):
            tab[prefix] = rng.standard_normal(V) * temp
    return tab


def test_whole_step_enumeration_every_gamma():
    """V = 3, k = 2: run the oracle's verify step over all draft paths and a
    grid of uniforms; at every position reached, the emitted token must follow
    the target's conditional law, for every verification length gamma."""
    rng = np.random.default_rng(3)
    V, k, J = 3, 2, 12
    tgt = _toy_tables(rng, V, k + 1)
    drf = _toy_tables(rng, V, k)
    grid = (np.arange(J) + 0.5) / J
    for gamma in range(k + 1):
        # weight[prefix][y]: mass of emitting y right after the accepted prefix
        weight = {}
        for path in itertools.product(range(V), repeat=k):
            p_path = 1.0
            for i in range(k):
                p_path *= _softmax(drf[path[:i]])[path[i]]
            z_t = np.stack([tgt[path[:i]] for i in range(k + 1)])[None]
            z_d = np.stack([drf[path[:i]] for i in range(k)])[None]
            x = np.array([path])
            combos = list(itertools.product(grid, repeat=k + 1))   # (u_0..u_{k-1}, u')
            Bn = len(combos)
            ua = np.array([c[:k] for c in combos])
            us = np.repeat(np.array([c[k] for c in combos])[:, None], k + 1, axis=1)
            out = O.verify_sample(np.repeat(z_t, Bn, 0), np.repeat(z_d, Bn, 0),
                                  np.repeat(x, Bn, 0), gamma=np.full(Bn, gamma),
                                  uniforms=(ua, us))
            for j in range(Bn):
                n = out["n_accept"][j]
                toks = out["tokens"][j]
                assert n <= gamma and np.all(toks[:n] == path[:n]) and np.all(toks[n + 1:] == -1)
                weight.setdefault(path[:n], np.zeros(V))
                weight[path[:n]][toks[n]] += p_path / Bn
        # Mass reaching `prefix` as accepted prefix, then emitting y at that position:
        # either the draft proposed y there and it was accepted (that mass is booked
        # under the longer prefix), or something was sampled at that position.
        for prefix, wv in weight.items():
            L = len(prefix)
            reach = sum(v.sum() for pre, v in weight.items() if pre[:L] == prefix)
            emitted = wv.copy()
            for y in range(V):
                emitted[y] += sum(v.sum() for pre, v in weight.items()
                                  if len(pre) > L and pre[:L + 1] == prefix + (y,))
            assert np.allclose(emitted / reach, _softmax(tgt[prefix]), atol=2.5 / J), (gamma, prefix)


def test_identical_models_accept_everything_and_bonus_is_target():
    rng = np.random.default_rng(4)
    B, k, V = 64, 3, 6
    z = rng.standard_normal((B, k + 1, V)).astype(np.float32)
    x = rng.integers(0, V, size=(B, k))
    out = O.verify_sample(z, z[:, :k], x, seed=11, step=2)
    assert np.all(out["n_accept"] == k)
    assert np.array_equal(out["tokens"][:, :k], x)
    assert np.all(out["flags"] & O.FLAG_RESIDUAL_FALLBACK == 0)
    for b in range(B):
        _, up = philox.sv_uniforms(11, 2, b, k)
        pt = _softmax(z[b, k])
        assert out["tokens"][b, k] == int(np.searchsorted(np.cumsum(pt), float(up) * np.cumsum(pt)[-1],
                                                          side="right"))


def test_disjoint_supports_reject_first_and_residual_is_target():
    ninf = -np.inf
    z_t = np.array([[[0.0, 1.0, ninf, ninf], [0, 0, 0, 0]]])
    z_d = np.array([[[ninf, ninf, 0.5, 0.0]]])
    for tok in (2, 3):
        for seed in range(20):
            out = O.verify_sample(z_t, z_d, np.array([[tok]]), seed=seed)
            assert out["n_accept"][0] == 0 and out["tokens"][0, 0] in (0, 1)
            assert abs(out["W"][0] - 1.0) < 1e-15


def test_one_hot_target_is_deterministic():
    ninf = -np.inf
    z_t = np.array([[[ninf, 3.0, ninf], [ninf, ninf, 0.0]]])
    z_d = np.array([[[0.0, 0.0, 0.0]]])
    for tok, seed in itertools.product(range(3), range(10)):
        out = O.verify_sample(z_t, z_d, np.array([[tok]]), seed=seed)
        if tok == 1:
            assert list(out["tokens"][0]) == [1, 2] and out["n_accept"][0] == 1
        else:
            assert list(out["tokens"][0]) == [1, -1] and out["n_accept"][0] == 0


def test_gamma_zero_draws_from_target_and_packed_equals_dense():
    rng = np.random.default_rng(5)
    B, k, V = 5, 4, 11
    z_t = (2 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    z_d = (z_t[:, :k] + rng.standard_normal((B, k, V))).astype(np.float32)
    x = rng.integers(0, V, size=(B, k))
    gamma = np.array([0, 4, 2, 1, 3])
    dense = O.verify_sample(z_t, z_d, x, gamma=gamma, seed=5)
    assert dense["n_accept"][0] == 0 and dense["tokens"][0, 0] >= 0
    assert np.all(dense["n_accept"] <= gamma)
    offs = np.concatenate([[0], np.cumsum(gamma + 1)])
    packed = np.concatenate([z_t[b, :gamma[b] + 1] for b in range(B)])
    out = O.verify_sample(packed, z_d, x, gamma=gamma, t_offsets=offs, seed=5)
    assert np.array_equal(out["tokens"], dense["tokens"])
    assert np.array_equal(out["n_accept"], dense["n_accept"])


def test_empirical_acceptance_rate_with_philox_uniforms():
    rng = np.random.default_rng(6)
    V, B = 16, 20000
    zt = rng.standard_normal(V) * 2
    zd = zt + rng.standard_normal(V)
    pd, pt = _softmax(zd), _softmax(zt)
    x = rng.choice(V, size=(B, 1), p=pd)
    z_t = np.broadcast_to(np.stack([zt, zt])[None], (B, 2, V))
    z_d = np.broadcast_to(zd[None, None], (B, 1, V))
    out = O.verify_sample(z_t, z_d, x, seed=99)
    rate = out["n_accept"].mean()
    expect = np.minimum(pt, pd).sum()
    assert abs(rate - expect) < 4 * np.sqrt(expect * (1 - expect) / B)
    # first emitted token follows the target (chi-square, V - 1 dof)
    counts = np.bincount(out["tokens"][:, 0], minlength=V)
    chi2 = ((counts - B * pt) ** 2 / (B * pt)).sum()
    assert chi2 < 45.0          # 99.99th percentile of chi2(15) is ~44.3


def test_flags_near_tie_residual_fallback_bad_inputs():
    # near tie: choose rho so that it sits 5e-7 above the accept uniform
    u, _ = philox.sv_uniforms(0, 0, 0, 0)
    u = float(u)
    rho = u + 5e-7
    z_t = np.array([[[np.log(rho), np.log(1 - rho) if rho < 1 else -50.0], [0.0, 0.0]]])
    z_d = np.array([[[0.0, -np.inf]]])
    out = O.verify_sample(z_t, z_d, np.array([[0]]), seed=0)
    assert out["flags"][0] & O.FLAG_NEAR_TIE and out["n_accept"][0] == 1
    # identical rows but an (impossible) reject forced by u = 1: residual mass 0 -> fallback
    z = np.array([[[0.0, 1.0, 2.0], [0.0, 0.0, 0.0]]])
    out = O.verify_sample(z, z[:, :1], np.array([[1]]),
                          uniforms=(np.array([[1.0]]), np.array([[0.5, 0.5]])))
    assert out["n_accept"][0] == 0 and out["flags"][0] & O.FLAG_RESIDUAL_FALLBACK
    pt = _softmax(z[0, 0])
    assert out["tokens"][0, 0] == int(np.searchsorted(np.cumsum(pt), 0.5 * np.cumsum(pt)[-1], side="right"))
    # NaN in the target row that must be sampled: no token, flagged
    zb = z.copy()
    zb[0, 0, 0] = np.nan
    out = O.verify_sample(zb, z[:, :1], np.array([[1]]), seed=1)
    assert out["flags"][0] & O.FLAG_BAD_ROW and out["n_accept"][0] == 0 and out["tokens"][0, 0] == -1
    # token id out of range: rejected there, flagged, residual still drawn
    out = O.verify_sample(z, z[:, :1], np.array([[7]]), seed=1)
    assert out["flags"][0] & O.FLAG_BAD_TOKEN and out["n_accept"][0] == 0 and out["tokens"][0, 0] >= 0


def test_residual_is_drawn_for_any_positive_mass():
    """The speculative-sampling rule has no floor: a residual of any mass W > 0 is drawn from
    (W = 0 exactly is the only fallback).  Two-token rows: P_t = (a, 1-a), P_d = (a-d, 1-a+d)
    give the residual (d, 0) exactly, mass d; d is walked down through 1e-6 (where single
    precision stops resolving it) to 1e-14."""
    a = 0.4
    for d in (1e-1, 1e-3, 3e-6, 1.1e-6, 0.9e-6, 2e-7, 1e-9, 1e-12, 1e-14):
        zt = np.log(np.array([a, 1 - a]))
        zd = np.log(np.array([a - d, 1 - a + d]))
        w, W, fl = O.sampling_weights(zt, zd)
        assert fl == 0, d
        assert abs(W - d) <= 1e-15 + 1e-12 * d and w[1] == 0.0 and w[0] == W
        for u in (0.01, 0.5, 0.99):
            assert O.inverse_cdf(w, W, u)[0] == 0
    # W = 0 exactly: nothing to draw from, the target row is used and flagged
    zt = np.log(np.array([a, 1 - a]))
    w, W, fl = O.sampling_weights(zt, zt.copy())
    assert fl == O.FLAG_RESIDUAL_FALLBACK and np.allclose(w, [a, 1 - a], rtol=1e-12) and abs(W - 1) < 1e-12


def test_emitted_law_is_the_target_for_nearly_equal_models():
    """Pins the no-floor rule by what it must achieve, not by a constant: with P_d within
    1e-2 ... 1e-12 of P_t (residual mass of that order) one verified position still emits
    exactly P_t:  sum_x P_d(x) [a(x) 1{x=y} + (1 - a(x)) r(y)] = P_t(y),  V <= 8.
    A rule that swapped a small residual for P_t would be off by about W^2 in the tokens that
    lose mass, which the tolerance (1e-3 of W^2) resolves down to W = 1e-6 in float64."""
    rng = np.random.default_rng(11)
    for V in (2, 3, 8):
        for eps in (1e-2, 1e-4, 1e-6):
            zt = rng.standard_normal(V) * 2
            zd = zt + eps * rng.standard_normal(V)
            pt, pd = _softmax(zt), _softmax(zd)
            w, W, fl = O.sampling_weights(zt, zd)
            assert fl == 0 and 0 < W < 4 * eps
            a = np.array([min(1.0, O.accept_ratio(zt, zd, t)[0]) for t in range(V)])
            emitted = pd * a + np.sum(pd * (1 - a)) * w / W
            assert np.max(np.abs(emitted - pt)) < max(1e-3 * W * W, 4e-16), (V, eps)
            # the same law with the target row in place of the residual is visibly wrong
            wrong = pd * a + np.sum(pd * (1 - a)) * pt
            assert np.max(np.abs(wrong - pt)) > 0.05 * W * W
        for eps in (1e-9, 1e-12):     # below float64's W^2 resolution: the residual's support
            zt = rng.standard_normal(V) * 2
            zd = zt + eps * rng.standard_normal(V)
            pt, pd = _softmax(zt), _softmax(zd)
            w, W, fl = O.sampling_weights(zt, zd)
            assert fl == 0 and W > 0
            assert np.array_equal(w > 0, pt > pd)


def test_admissible_sets_with_an_absolute_band():
    """The comparison aid of inverse_cdf: an absolute band widens the admissible set (and only
    that); tokens outside `support` are never admissible, tokens of zero weight inside it are."""
    w = np.array([0.25, 0.0, 0.5, 0.25, 0.0])
    support = np.array([True, True, True, True, False])
    y0, m0, adm0 = O.inverse_cdf(w, 1.0, 0.2499)
    y1, m1, adm1 = O.inverse_cdf(w, 1.0, 0.2499, abs_band=1e-3, support=support)
    assert (y0, m0) == (y1, m1) and list(adm0) == [0] and list(adm1) == [0, 1, 2]
    # a residual far below the band: every supported token is admissible
    w = np.array([0.0, 3e-9, 0.0, 1e-9, 0.0])
    y, _, adm = O.inverse_cdf(w, 4e-9, 0.9, abs_band=1e-6, support=support)
    assert y == 3 and list(adm) == [0, 1, 2, 3]
    z = np.array([[[0.0, 1.0, 2.0], [0.0, 0.0, 0.0]]])
    r0 = O.verify_sample(z, z[:, :1] + 0.3, np.array([[1]]), seed=4)
    r1 = O.verify_sample(z, z[:, :1] + 0.3, np.array([[1]]), seed=4, cdf_abs_band=0.5)
    for name in ("tokens", "n_accept", "ratio", "margin", "W", "resid"):
        assert np.array_equal(r0[name], r1[name], equal_nan=True), name
    assert r1["flags"][0] & O.FLAG_NEAR_CDF_EDGE and not (r0["flags"][0] & O.FLAG_NEAR_CDF_EDGE)

