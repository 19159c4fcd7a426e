"""Pins for the sampling-warp oracle (CPU only)."""
import numpy as np
import scipy.special
import torch

from oracle import sv_oracle as O
from oracle import warp_oracle as W


def _distinct_row(rng, V, scale=3.0):
    z = scale * rng.standard_normal(V)
    assert np.unique(z).size == V
    return z


def test_top_k_matches_torch_topk_without_ties():
    rng = np.random.default_rng(0)
    for V, K in ((50, 1), (50, 7), (1000, 20), (1000, 999)):
        z = _distinct_row(rng, V)
        cut, fl = W.warp_cutoff(z, 1.0, K, 1.0)
        vals, idx = torch.topk(torch.from_numpy(z), K)
        assert fl == 0 and cut == float(vals[-1])
        assert set(np.nonzero(z >= cut)[0]) == set(idx.tolist())
    z = _distinct_row(rng, 30)
    for K in (0, 30, 31, -2):
        assert W.warp_cutoff(z, 1.0, K, 1.0)[0] == -np.inf       # off


def test_top_p_matches_sort_cumsum_without_ties():
    rng = np.random.default_rng(1)
    for V, T, P in ((40, 1.0, 0.9), (500, 0.7, 0.8), (500, 0.6, 0.95), (2000, 1.3, 0.5), (10, 1.0, 1e-9)):
        z = _distinct_row(rng, V)
        cut, fl = W.warp_cutoff(z, T, 0, P)
        p = torch.softmax(torch.from_numpy(z) / T, 0)
        srt, order = torch.sort(p, descending=True)
        csum = torch.cumsum(srt, 0)
        n_keep = int((csum < P).sum()) + 1                      # tokens until the mass reaches P
        assert set(np.nonzero(z >= cut)[0]) == set(order[:n_keep].tolist())
        kept_mass = float(p[torch.from_numpy(z >= cut)].sum())
        assert kept_mass >= P - 1e-12
        assert kept_mass - float(srt[n_keep - 1]) < P + 1e-12   # minimal: dropping the last one falls short


def test_top_k_then_top_p_order_and_renormalisation():
    rng = np.random.default_rng(2)
    z = _distinct_row(rng, 300)
    T, K, P = 0.7, 20, 0.8
    cut, _ = W.warp_cutoff(z, T, K, P)
    vals, idx = torch.topk(torch.from_numpy(z), K)
    p = torch.softmax(vals / T, 0)                              # top-p sees the top-k survivors only
    csum = torch.cumsum(p, 0)
    n_keep = int((csum < P).sum()) + 1
    assert cut == float(vals[n_keep - 1])
    # top-p alone would keep a different set when the tail beyond K carries mass
    cut_p_only, _ = W.warp_cutoff(z, T, 0, P)
    assert cut_p_only <= cut


def test_ties_are_kept_or_dropped_together():
    z = np.array([3.0, 1.0, 3.0, 2.0, 2.0, 2.0, 0.0, -1.0])
    assert W.warp_cutoff(z, 1.0, 1, 1.0)[0] == 3.0               # both 3.0 entries stay
    assert W.warp_cutoff(z, 1.0, 3, 1.0)[0] == 2.0               # third largest is a 2.0: all three 2.0 stay
    assert W.warp_cutoff(z, 1.0, 5, 1.0)[0] == 2.0
    p = scipy.special.softmax(z)
    top = p[z == 3.0].sum()
    assert W.warp_cutoff(z, 1.0, 0, top - 1e-3)[0] == 3.0
    assert W.warp_cutoff(z, 1.0, 0, top + 1e-3)[0] == 2.0        # needs the whole 2.0 group
    cut, fl = W.warp_cutoff(z, 1.0, 0, float(top))
    assert fl & O.FLAG_NEAR_TIE                                   # deciding mass sits on P


def test_monotone_in_k_and_p_and_bf16_rows():
    rng = np.random.default_rng(3)
    t = torch.from_numpy(2.5 * rng.standard_normal(4000)).to(torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    prev = np.inf
    for K in (1, 5, 50, 500, 3999):
        c = W.warp_cutoff(bits, 1.0, K, 1.0)[0]
        assert c <= prev and (O.upcast(bits) >= c).sum() >= K
        prev = c
    prev = np.inf
    for P in (0.1, 0.5, 0.9, 0.99, 0.999999):
        c = W.warp_cutoff(bits, 0.7, 0, P)[0]
        assert c <= prev
        prev = c


def test_warp_rows_and_temperature():
    rng = np.random.default_rng(4)
    z = (2 * rng.standard_normal((2, 3, 64))).astype(np.float32)
    out, cut, fl = W.warp_rows(z, 0.6, 10, 0.9)
    assert out.shape == z.shape and cut.shape == (2, 3) and not fl.any()
    for idx in np.ndindex(2, 3):
        keep = z[idx].astype(np.float64) >= cut[idx]
        assert np.all(np.isneginf(out[idx][~keep])) and np.allclose(out[idx][keep], z[idx][keep] / 0.6)
        lse, lp = O.log_softmax_row(out[idx])
        ref = scipy.special.softmax(z[idx][keep].astype(np.float64) / 0.6)
        assert np.allclose(np.exp(lp[keep]), ref, rtol=1e-12) and 1 <= keep.sum() <= 10
    # no warp: identity up to the cast
    out, cut, _ = W.warp_rows(z, 1.0, 0, 1.0)
    assert np.array_equal(out, z.astype(np.float64)) and np.all(np.isneginf(cut))
    # bad rows are flagged and passed through
    zb = z.copy()
    zb[0, 0, 3] = np.nan
    out, cut, fl = W.warp_rows(zb, 1.0, 5, 0.9)
    assert fl[0, 0] & O.FLAG_BAD_ROW and np.isnan(cut[0, 0]) and np.isnan(out[0, 0, 3])
