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


def test_warps_in_sequence_match_the_transformers_logits_processors():
    """Temperature -> top-k -> top-p on rows without ties: the kept set of the oracle is the set
    the `transformers` warpers leave finite, and the kept values are z / T."""
    from transformers import TemperatureLogitsWarper, TopKLogitsWarper, TopPLogitsWarper
    rng = np.random.default_rng(11)
    ids = torch.zeros((1, 1), dtype=torch.long)
    for V, T, K, P in ((200, 0.7, 20, 0.8), (1000, 0.95, 20, 0.6), (1000, 0.6, 0, 0.9), (64, 1.3, 5, 1.0),
                       (5000, 0.7, 50, 0.95), (300, 1.0, 0, 0.5)):
        for _ in range(5):
            z = _distinct_row(rng, V)
            y, cut, fl = W.warp_rows(z[None, None, :], T, K, P)
            s = torch.from_numpy(z)[None, :].clone()
            s = TemperatureLogitsWarper(T)(ids, s)
            if 0 < K < V:
                s = TopKLogitsWarper(top_k=K)(ids, s)
            if P < 1.0:
                s = TopPLogitsWarper(top_p=P)(ids, s)
            lib_kept = np.isfinite(s[0].numpy())
            if fl[0, 0] & O.FLAG_NEAR_TIE:
                continue                                      # a decision within 1e-6 of P may go either way
            mine = np.isfinite(y[0, 0])
            assert np.array_equal(mine, lib_kept), (V, T, K, P, mine.sum(), lib_kept.sum())
            assert np.allclose(y[0, 0][mine], s[0].numpy()[lib_kept], rtol=1e-12)


def test_repetition_penalty_matches_the_transformers_processor():
    from transformers import RepetitionPenaltyLogitsProcessor
    rng = np.random.default_rng(12)
    for V, n_hist, theta in ((50, 7, 1.3), (1000, 200, 1.1), (1000, 40, 1.05), (33, 60, 2.0), (200, 0, 1.2)):
        B, R = 3, 2
        z = (3 * rng.standard_normal((B, R, V))).astype(np.float32)
        z[0, 0, 3] = 0.0
        z[1, 1, 5] = -np.inf
        hist = rng.integers(0, V, size=(B, max(n_hist, 1))).astype(np.int64)
        if n_hist == 0:
            hist[:] = -1                                     # padding only
        else:
            hist[:, 0] = hist[:, -1]                         # a duplicate: penalised once
            hist[0, 1] = 3
            hist[1, 2] = 5
        got = W.repetition_penalty(z, hist, theta)
        proc = RepetitionPenaltyLogitsProcessor(penalty=float(np.float32(theta)))
        for i in range(R):
            if n_hist == 0:
                ref = z[:, i]
            else:
                ref = proc(torch.from_numpy(hist), torch.from_numpy(z[:, i].copy())).numpy()
            assert np.array_equal(got[:, i], ref, equal_nan=True), (V, n_hist, theta, i)
    # padding and out-of-range ids are ignored, theta = 1 changes nothing
    z = (3 * rng.standard_normal((1, 1, 20))).astype(np.float32)
    assert np.array_equal(W.repetition_penalty(z, np.array([[-1, 20, 99, -7]]), 1.5), z)
    assert np.array_equal(W.repetition_penalty(z, np.array([[1, 2, 3]]), 1.0), z)


def test_repetition_penalty_draft_prefix_and_bfloat16_storage():
    rng = np.random.default_rng(13)
    B, k, V = 2, 3, 40
    zf = (3 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    zb = torch.from_numpy(zf).to(torch.bfloat16)
    bits = zb.view(torch.int16).numpy().view(np.uint16)
    hist = np.array([[1, 2, -1], [7, 7, 9]])
    x = np.array([[4, 5, 6], [9, 10, 11]])
    theta = 1.25
    got = W.repetition_penalty(bits, hist, theta, x=x)
    stored = zb.float().numpy()
    for b in range(B):
        for i in range(k + 1):
            toks = {int(t) for t in hist[b] if t >= 0} | {int(t) for t in x[b, :min(i, k)]}
            exp = stored[b, i].copy()
            for t in toks:                                   # position i sees the tokens drafted before it
                v = np.float32(exp[t])
                exp[t] = v * np.float32(theta) if v < 0 else v / np.float32(theta)
            exp_bits = torch.from_numpy(exp).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
            assert np.array_equal(got[b, i], exp_bits), (b, i)
    # the rounding helper against torch's conversion on arbitrary float32 values (ties, tiny, huge, inf)
    v = np.concatenate([rng.standard_normal(5000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 5000),
                        np.array([0.0, -0.0, np.inf, -np.inf, 1.00390625, 1.01171875, 3.3895e38], dtype=np.float32)])
    mine = W._store_like(v, np.zeros(1, dtype=np.uint16))
    ref = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(mine, ref)
