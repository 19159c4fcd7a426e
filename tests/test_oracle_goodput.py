"""Pins for the oracle's estimator comparison and goodput bookkeeping (CPU only)."""
import numpy as np
import scipy.special
import scipy.stats

import svgen
from oracle import goodput_oracle as GO
from oracle import profile_oracle as PO
from oracle import sv_oracle as O


def _batch(seed, B=6, k=3, V=300, idx=3):
    c = svgen.make_config(idx, seed=seed, B=B, k=k, V=V, dtype="f32")
    return tuple(svgen.to_numpy_bits(c[n]) for n in ("z_t", "z_d", "z_c")) + (c["x"].numpy(),)


def test_signals_against_scipy():
    zt, zd, zc, x = _batch(1)
    sig = GO.signals(zd, zc, x)
    pd = scipy.special.softmax(zd.astype(np.float64), axis=-1)
    H = scipy.stats.entropy(pd, axis=-1)                       # nats
    px = np.take_along_axis(pd, x[..., None].astype(np.int64), axis=-1)[..., 0]
    assert np.allclose(sig["H_d"], H, rtol=1e-6) and np.allclose(sig["pd_x"], px, rtol=1e-6)
    pc = scipy.special.softmax(zc.astype(np.float64), axis=-1)
    assert np.allclose(sig["S"], np.minimum(pd, pc).sum(-1), rtol=1e-6)


def test_one_dimensional_profiles_are_cell_means_and_calibrated():
    rng = np.random.default_rng(5)
    n, V = 4000, 1000
    sig = dict(S=rng.random((n, 1)).astype(np.float32), A=rng.random((n, 1)).astype(np.float32),
               H_d=(rng.random((n, 1)) * np.log(V)).astype(np.float32),
               pd_x=rng.random((n, 1)).astype(np.float32) ** 3)
    # X depends on the entropy signal only
    ratio = np.clip(1.0 - sig["H_d"] / np.log(V) + 0.05 * rng.standard_normal((n, 1)), 0, 1.5).astype(np.float32)
    X = np.minimum(ratio, 1.0).astype(np.float64)
    profs = {m: GO.build_profile(m, sig, ratio, V, cells=16, n_x=8) for m in GO.ESTIMATORS}
    for m in ("entropy", "probability"):
        e1, e2, table, info = profs[m]
        assert table.shape == (16, 1) and list(e2) == [0.0, 1.0] and np.all(np.diff(e1) >= 0)
        a1 = GO.axes_of(m, sig)[0].ravel()
        # cell means by masking, with numpy's own binning of the same half-open cells
        cell = np.clip(np.searchsorted(e1, a1, side="right") - 1, 0, 15)
        for j in range(16):
            sel = cell == j
            assert sel.sum() >= n // 16 - 16                     # equal-count edges
            assert abs(table[j, 0] - X.ravel()[sel].mean()) < 1e-6
        p_hat, _ = GO.estimate(m, sig, profs[m])
        assert abs(p_hat.astype(np.float64).mean() - X.mean()) < 1e-6    # calibrated on its own samples
    # the informative signal wins, the uninformative ones carry next to nothing
    gain = {m: profs[m][3][2] for m in GO.ESTIMATORS}
    assert gain["entropy"] > 1.0 and gain["probability"] < 0.15 and gain["sv"] < 0.15
    # deterministic X given the cell: conditional entropy 0, gain = H(X)
    r2 = (np.floor(sig["pd_x"] * 4) / 4 + 0.1).astype(np.float32)
    e1, e2, table, info = GO.build_profile("probability", sig, r2, V, cells=4, n_x=4)
    cell_of = np.clip(np.searchsorted(e1, sig["pd_x"].ravel(), side="right") - 1, 0, 3)
    if all(len(set(r2.ravel()[cell_of == j])) == 1 for j in range(4)):
        assert abs(info[1]) < 1e-12 and abs(info[2] - info[0]) < 1e-12


def test_step_bookkeeping_closed_forms():
    zt, zd, zc, x = _batch(2)
    B, k, V = zd.shape
    ones = np.ones((4, 4), dtype=np.float32)
    e = np.linspace(0, 1, 5).astype(np.float32)
    flat = np.full(B * k + 1, 7.0, dtype=np.float32)            # verifying more costs nothing
    out, sig = GO.step(zt, zd, zc, x, {"sv": (e, e, ones)}, flat, seed=3, step_index=1)
    # estimates of 1 and a flat latency: everything is verified, i.e. plain SD
    assert np.array_equal(out["sv"]["gamma"], np.full(B, k)) and out["sv"]["M"] == B * k
    assert np.array_equal(out["sv"]["n_accept"], out["sd"]["n_accept"])
    ref = O.verify_sample(zt, zd, x, seed=3, step=1)
    assert np.array_equal(out["sd"]["n_accept"], ref["n_accept"])
    assert out["sd"]["accepted"] == int(ref["n_accept"].sum()) and out["sd"]["verified"] == B * k
    # a latency that explodes after the first token: exactly one token is verified
    steep = np.concatenate(([1.0, 1.0], np.full(B * k - 1, 1e9))).astype(np.float32)
    out2, _ = GO.step(zt, zd, zc, x, {"sv": (e, e, ones)}, steep, seed=3, step_index=1)
    assert out2["sv"]["M"] == 1 and out2["sv"]["gamma"].sum() == 1 and out2["sv"]["latency"] == 1.0
    assert out2["sv"]["accepted"] <= 1
    # identical target and draft: every verified token is accepted
    out3, _ = GO.step(np.concatenate([zd, zd[:, :1]], axis=1), zd, zc, x, {"sv": (e, e, ones)}, flat, 3, 1)
    assert out3["sd"]["accepted"] == B * k
    tot = GO.totals([out, out3])
    assert tot["sd"]["accepted"] == out["sd"]["accepted"] + B * k and tot["sd"]["verified"] == 2 * B * k
    assert abs(tot["sd"]["goodput"] - tot["sd"]["accepted"] / 14.0) < 1e-12
    assert abs(tot["sd"]["accept_rate"] - tot["sd"]["accepted"] / (2 * B * k)) < 1e-12
    assert tot["sv"]["mean_verified_per_seq"] == k


def test_companion_signal_is_the_most_informative_on_the_synthetic_recipe():
    """The synthetic recipes give draft and companion independent noise around the target, so
    their agreement says how far the draft is from the target; the draft's own entropy and token
    probability say much less.  (The direction of the paper's comparison, not its numbers.)"""
    zt, zd, zc, x = _batch(4, B=48, k=4, V=2000)
    sig = GO.signals(zd, zc, x)
    ratio, _ = PO.accept_probability_ratio(zt, zd, x)
    gain = {m: GO.build_profile(m, sig, ratio, 2000, cells=16, n_x=8)[3][2] for m in GO.ESTIMATORS}
    assert gain["sv"] > gain["entropy"] and gain["sv"] > gain["probability"], gain
