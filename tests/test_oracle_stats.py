"""Pins for the oracle's row normalisers, S, A, divergences and the binned
estimate (CPU only).  Every check is against something the oracle did not
produce itself: a library routine, a closed form, an invariant."""
import numpy as np
import scipy.special
import torch

from oracle import sv_oracle as O


def _rows(rng, B, k, V, scale=2.0):
    return (scale * rng.standard_normal((B, k, V))).astype(np.float32)


def test_upcast_bf16_is_exact():
    t = torch.randn(1000, dtype=torch.float32).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(O.upcast(bits), t.to(torch.float64).numpy())


def test_lse_matches_scipy_and_torch():
    rng = np.random.default_rng(0)
    for V in (1, 2, 7, 1000, 32000):
        z = (3 * rng.standard_normal(V)).astype(np.float32).astype(np.float64)
        lse, lp = O.log_softmax_row(z)
        assert abs(lse - scipy.special.logsumexp(z)) < 1e-12 * max(1, abs(lse))
        ref = torch.log_softmax(torch.from_numpy(z), dim=0).numpy()
        assert np.allclose(lp, ref, rtol=0, atol=1e-12)
        assert abs(np.exp(lp).sum() - 1.0) < 1e-12


def test_lse_shift_and_neg_inf():
    rng = np.random.default_rng(1)
    z = rng.standard_normal(500)
    lse, _ = O.log_softmax_row(z)
    lse2, _ = O.log_softmax_row(z + 37.5)
    assert abs(lse2 - lse - 37.5) < 1e-12
    z2 = np.concatenate([z, np.full(20, -np.inf)])
    lse3, lp3 = O.log_softmax_row(z2)
    assert abs(lse3 - lse) < 1e-13 and np.all(lp3[-20:] == -np.inf)
    # huge logits do not overflow
    lse4, _ = O.log_softmax_row(np.array([1e4, 1e4]))
    assert abs(lse4 - (1e4 + np.log(2))) < 1e-9


def test_bad_rows_give_nan():
    for bad in (np.array([0.0, np.nan, 1.0]), np.full(4, -np.inf), np.array([0.0, np.inf])):
        lse, lp = O.log_softmax_row(bad)
        assert np.isnan(lse) and np.all(np.isnan(lp))


def test_S_equals_library_min_of_softmaxes_and_is_symmetric():
    rng = np.random.default_rng(2)
    zd = _rows(rng, 2, 3, 257)
    zc = (zd + rng.standard_normal(zd.shape)).astype(np.float32)
    x = rng.integers(0, 257, size=(2, 3))
    r = O.row_stats(zd, zc, x)
    pd = torch.softmax(torch.from_numpy(zd).double(), -1)
    pc = torch.softmax(torch.from_numpy(zc).double(), -1)
    S_ref = torch.minimum(pd, pc).sum(-1).numpy()
    assert np.allclose(r["S"], S_ref, rtol=1e-12)
    assert np.all((r["S"] > 0) & (r["S"] <= 1 + 1e-15))
    assert np.allclose(r["TV"], 0.5 * (pd - pc).abs().sum(-1).numpy(), atol=1e-12)
    r2 = O.row_stats(zc, zd, x)
    assert np.allclose(r["S"], r2["S"], rtol=1e-14)
    import scipy.stats
    assert np.allclose(r["H_d"], scipy.stats.entropy(pd.numpy(), axis=-1), rtol=1e-12)
    for b in range(2):
        for i in range(3):
            assert abs(r["pd_x"][b, i] - float(pd[b, i, x[b, i]])) < 1e-15
    kl_ref = (pd * (pd.log() - pc.log())).sum(-1).numpy()
    assert np.allclose(r["KL"], kl_ref, rtol=1e-10)
    assert np.all(r["KL"] >= 0)
    # A against an independent evaluation through probabilities
    for b in range(2):
        for i in range(3):
            t = x[b, i]
            assert abs(r["A"][b, i] - min(1.0, float(pc[b, i, t] / pd[b, i, t]))) < 1e-12


def test_identical_and_shifted_rows():
    rng = np.random.default_rng(3)
    zd = _rows(rng, 1, 4, 100)
    x = rng.integers(0, 100, size=(1, 4))
    for zc in (zd.copy(), (zd.astype(np.float64) + 3.0)):
        r = O.row_stats(zd, zc, x)
        assert np.allclose(r["S"], 1.0, atol=1e-12)
        assert np.allclose(r["A"], 1.0, atol=1e-12)
        assert np.allclose(r["TV"], 0.0, atol=1e-12)
        assert np.allclose(r["KL"], 0.0, atol=1e-12)


def test_two_token_closed_form():
    # V = 2: P = (sigmoid(a), 1 - sigmoid(a)); S = min(p, q) + min(1-p, 1-q) = 1 - |p - q|
    for a, c in ((0.3, -1.2), (2.0, 2.5), (-4.0, 4.0)):
        zd = np.array([[[a, 0.0]]], dtype=np.float64)
        zc = np.array([[[c, 0.0]]], dtype=np.float64)
        p = 1 / (1 + np.exp(-a))
        q = 1 / (1 + np.exp(-c))
        r = O.row_stats(zd, zc, np.array([[0]]))
        assert abs(r["S"][0, 0] - (1 - abs(p - q))) < 1e-14
        assert abs(r["A"][0, 0] - min(1, q / p)) < 1e-14


def test_mean_of_A_under_draft_is_S():
    # E_{x ~ P_d} min(1, P_c(x)/P_d(x)) = sum_v min(P_d, P_c): ties A to S.
    rng = np.random.default_rng(4)
    V = 50
    zd = _rows(rng, 1, 1, V)
    zc = (zd + 1.5 * rng.standard_normal(zd.shape)).astype(np.float32)
    pd = scipy.special.softmax(zd[0, 0].astype(np.float64))
    acc = 0.0
    for t in range(V):
        r = O.row_stats(zd, zc, np.array([[t]]))
        acc += pd[t] * r["A"][0, 0]
    assert abs(acc - r["S"][0, 0]) < 1e-12


def test_zero_draft_probability_token_and_bad_inputs():
    zd = np.array([[[0.0, -np.inf, 1.0]]])
    zc = np.array([[[0.0, 0.5, 1.0]]])
    r = O.row_stats(zd, zc, np.array([[1]]))
    assert r["A"][0, 0] == 1.0 and r["flags"][0, 0] == 0
    assert np.isfinite(r["KL"][0, 0])          # the P_d(v) = 0 entry is skipped
    r = O.row_stats(zd, zc, np.array([[3]]))
    assert np.isnan(r["A"][0, 0]) and r["flags"][0, 0] & O.FLAG_BAD_TOKEN
    zd2 = zd.copy()
    zd2[0, 0, 0] = np.nan
    r = O.row_stats(zd2, zc, np.array([[0]]))
    assert r["flags"][0, 0] & O.FLAG_BAD_ROW and np.isnan(r["S"][0, 0])


# ------------------------------------------------------------------ estimate
def test_accept_estimate_matches_searchsorted_and_closes_top_bin():
    rng = np.random.default_rng(5)
    edges_s = np.array([0, 0.2, 0.5, 0.55, 0.9, 1.0], dtype=np.float32)
    edges_a = np.array([0, 0.1, 0.3, 1.0], dtype=np.float32)
    table = rng.random((5, 3)).astype(np.float32)
    S = rng.random(500).astype(np.float32)
    A = rng.random(500).astype(np.float32)
    S[:6] = edges_s            # exactly on edges, including both ends
    A[:4] = edges_a
    S[6], A[6] = 1.0, 1.0      # saturated values belong to the last bin
    S[7], A[7] = -0.5, 1.5     # outside: clamp
    p, flag = O.accept_estimate(S, A, edges_s, edges_a, table)
    i_s = np.clip(np.searchsorted(edges_s, S, side="right") - 1, 0, 4)
    i_a = np.clip(np.searchsorted(edges_a, A, side="right") - 1, 0, 2)
    assert np.array_equal(p, table[i_s, i_a])
    assert p[6] == table[4, 2]
    assert p[7] == table[0, 2]
    # a value on an interior edge belongs to the upper bin (half-open on the right)
    assert i_s[1] == 1 and p[1] == table[1, i_a[1]]
    assert flag[1] == 1 and flag[2] == 1
    far = (np.min(np.abs(S[:, None] - edges_s[None, 1:-1]), 1) > 1e-4) & \
          (np.min(np.abs(A[:, None] - edges_a[None, 1:-1]), 1) > 1e-4)
    assert np.all(flag[far] == 0)


def test_accept_estimate_nan_goes_to_first_bin_flagged():
    edges = np.linspace(0, 1, 6).astype(np.float32)
    table = np.arange(25, dtype=np.float32).reshape(5, 5)
    p, flag = O.accept_estimate(np.array([np.nan], np.float32), np.array([0.5], np.float32),
                                edges, edges, table)
    assert p[0] == table[0, 2] and flag[0] == 1
