"""Pins for the profile-construction / information-gain oracle (CPU only)."""
import numpy as np
import scipy.stats

from oracle import profile_oracle as P
from oracle import sv_oracle as O


def test_accumulate_matches_histogramdd_and_cell_means():
    rng = np.random.default_rng(0)
    n = 3000
    S = rng.random(n).astype(np.float32)
    A = np.minimum(1, 1.4 * rng.random(n)).astype(np.float32)      # saturates at 1 like the real A
    X = (1.6 * rng.random(n)).astype(np.float32)                   # ratios above 1 clip to 1
    S[:5] = [0.0, 1.0, 0.2, 0.4, np.nan]
    edges_s = np.array([0, 0.2, 0.4, 0.7, 1.0], np.float32)
    edges_a = np.linspace(0, 1, 6).astype(np.float32)
    n_x = 8
    counts, sum_x = P.accumulate(S, A, X, edges_s, edges_a, n_x)
    ok = ~np.isnan(S)
    Xc = np.clip(X, 0, 1)
    ref, _ = np.histogramdd(np.stack([S[ok], A[ok], Xc[ok]], 1),
                            bins=[edges_s.astype(np.float64), edges_a.astype(np.float64),
                                  np.linspace(0, 1, n_x + 1)])
    assert np.array_equal(counts, ref.astype(np.int64))
    assert counts.sum() == ok.sum()
    i_s = np.clip(np.searchsorted(edges_s, S, side="right") - 1, 0, 3)
    i_a = np.clip(np.searchsorted(edges_a, A, side="right") - 1, 0, 4)
    for a in range(4):
        for b in range(5):
            m = ok & (i_s == a) & (i_a == b)
            assert abs(sum_x[a, b] - Xc[m].astype(np.float64).sum()) < 1e-9
    # accumulating in two batches equals one batch
    c2, s2 = P.accumulate(S[:1000], A[:1000], X[:1000], edges_s, edges_a, n_x)
    c2, s2 = P.accumulate(S[1000:], A[1000:], X[1000:], edges_s, edges_a, n_x, c2, s2)
    assert np.array_equal(c2, counts) and np.allclose(s2, sum_x, rtol=1e-13)


def test_x_bin_top_closed_and_float32_decision():
    assert P.x_bin(1.0, 10) == 9 and P.x_bin(7.5, 10) == 9 and P.x_bin(0.0, 10) == 0
    assert P.x_bin(-0.3, 10) == 0 and P.x_bin(np.nan, 10) == -1
    assert P.x_bin(0.3, 10) == int(np.floor(np.float32(np.float32(0.3) * np.float32(10))))
    assert P.x_bin(0.25, 4) == 1 and P.x_bin(np.nextafter(np.float32(0.25), np.float32(0)), 4) == 0


def test_entropies_against_scipy_and_closed_forms():
    rng = np.random.default_rng(1)
    counts = rng.integers(0, 50, size=(4, 5, 6))
    counts[1, 2] = 0                                   # an empty cell
    sum_x = rng.random((4, 5)) * counts.sum(2)
    table, (h_x, h_c, ig) = P.finalize(counts, sum_x)
    N = counts.sum()
    assert abs(h_x - scipy.stats.entropy(counts.sum((0, 1)), base=2)) < 1e-12
    ref = sum(counts[i, j].sum() / N * scipy.stats.entropy(counts[i, j], base=2)
              for i in range(4) for j in range(5) if counts[i, j].sum() > 0)
    assert abs(h_c - ref) < 1e-12 and abs(ig - (h_x - h_c)) < 1e-15
    assert ig >= -1e-12                                # conditioning never increases entropy
    # mutual information through the joint distribution: I = H(X) + H(Y) - H(X,Y)
    cell = counts.sum(2).ravel()
    joint = counts.reshape(-1, 6)
    mi = scipy.stats.entropy(counts.sum((0, 1)), base=2) + scipy.stats.entropy(cell, base=2) \
        - scipy.stats.entropy(joint.ravel(), base=2)
    assert abs(ig - mi) < 1e-12
    # table: cell means, empty cell -> global mean
    assert abs(table[0, 0] - sum_x[0, 0] / counts[0, 0].sum()) < 1e-6
    assert abs(table[1, 2] - sum_x.sum() / N) < 1e-6


def test_information_gain_extremes():
    # X independent of the cell: joint = outer product -> zero gain
    px = np.array([10, 20, 30, 40])
    cells = np.array([[1, 2], [3, 4]])
    counts = cells[:, :, None] * px[None, None, :]
    _, (h_x, h_c, ig) = P.finalize(counts, np.zeros((2, 2)))
    assert abs(ig) < 1e-12 and abs(h_x - scipy.stats.entropy(px, base=2)) < 1e-12
    # X a deterministic function of the cell: conditional entropy 0, gain = H(X) = 2 bits
    counts = np.zeros((2, 2, 4), dtype=np.int64)
    for j, idx in enumerate(np.ndindex(2, 2)):
        counts[idx][j] = 25
    _, (h_x, h_c, ig) = P.finalize(counts, np.zeros((2, 2)))
    assert abs(h_x - 2.0) < 1e-12 and abs(h_c) < 1e-12 and abs(ig - 2.0) < 1e-12
    # no samples at all
    table, info = P.finalize(np.zeros((3, 3, 5)), np.zeros((3, 3)))
    assert np.all(table == 0) and info == (0.0, 0.0, 0.0)


def test_quantile_edges_equal_counts():
    rng = np.random.default_rng(2)
    v = rng.random(1000).astype(np.float32) ** 2           # denser near 0 -> smaller bins there
    v[::50] = np.nan
    e = P.quantile_edges(v, 16)
    assert e[0] == 0 and e[-1] == 1 and np.all(np.diff(e) >= 0)
    assert np.all(np.diff(e)[:4] < np.diff(e)[-4:].min())  # adaptive: finer where dense
    good = v[~np.isnan(v)]
    srt = np.sort(good)
    for j in range(1, 16):
        assert e[j] == srt[(j * good.size) // 16]
    idx = np.array([O._bin_index(x, e) for x in good])
    per_bin = np.bincount(idx, minlength=16)
    assert per_bin.max() - per_bin.min() <= 2
    # heavy ties (A saturates at 1): edges stay ascending, empty bins are allowed
    a = np.minimum(1, 3 * rng.random(500)).astype(np.float32)
    e = P.quantile_edges(a, 17)
    assert np.all(np.diff(e) >= 0) and e[-1] == 1


def test_accept_probability_for_every_position():
    rng = np.random.default_rng(3)
    B, k, V = 3, 4, 50
    z_t = (2 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    z_d = (z_t[:, :k] + rng.standard_normal((B, k, V))).astype(np.float32)
    x = rng.integers(0, V, size=(B, k))
    x[1, 2] = V + 3
    ratio, flags = P.accept_probability_ratio(z_t, z_d, x)
    import scipy.special
    pt = scipy.special.softmax(z_t.astype(np.float64), -1)
    pd = scipy.special.softmax(z_d.astype(np.float64), -1)
    for b in range(B):
        for i in range(k):
            if (b, i) == (1, 2):
                assert np.isnan(ratio[b, i]) and flags[b, i] & O.FLAG_BAD_TOKEN
            else:
                assert abs(ratio[b, i] - pt[b, i, x[b, i]] / pd[b, i, x[b, i]]) < 1e-10 * ratio[b, i]
    # the mean of min(1, ratio) under x ~ P_d is the acceptance rate 1 - TV (ties X to verification)
    acc = sum(pd[0, 0, t] * min(1.0, P.accept_probability_ratio(z_t[:1, :1], z_d[:1, :1], np.array([[t]]))[0][0, 0])
              for t in range(V))
    assert abs(acc - np.minimum(pt[0, 0], pd[0, 0]).sum()) < 1e-12
