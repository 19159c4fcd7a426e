"""GPU parity of the compacted-support path (sv_warp_compact, sv_row_stats_sparse,
sv_verify_sample_sparse) against the oracle: the oracle warps whole rows
(oracle/warp_oracle.warp_rows) and runs the ordinary dense row_stats /
verify_sample on them; the GPU works on the few kept tokens only."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O
from oracle import warp_oracle as W

import harness as H

pytestmark = pytest.mark.gpu

SERIES = [(0.7, 20, 0.8), (0.95, 20, 0.6), (0.6, 0, 0.9)]      # the paper's table of sampling hyper-parameters
NOT_COMPACT = 32


def _t32(T):
    return float(np.float32(T))


def _compact(z, T, K, Pp, cap):
    P = H.sv()
    rows = z.numel() // z.shape[-1]
    sup = P.Supports(rows, cap)
    sup.count.fill_(-77)
    sup.token.fill_(-3)
    sup.prob.fill_(-1.0)
    cut = torch.full((rows,), 123.0, dtype=torch.float32, device="cuda")
    flags = torch.full((rows,), 99, dtype=torch.int32, device="cuda")
    P.sv_warp_compact(z, T, K, Pp, sup, cut, flags)
    torch.cuda.synchronize()
    return sup, cut.cpu().numpy(), flags.cpu().numpy().astype(np.uint32)


def _check_supports(z_torch, T, K, Pp, cap):
    """Every compact row lists exactly the oracle's kept tokens with their probabilities."""
    zn = svgen.to_numpy_bits(z_torch)
    V = zn.shape[-1]
    rows = zn.reshape(-1, V)
    sup, cut, gflags = _compact(z_torch.cuda(), T, K, Pp, cap)
    count = sup.count.cpu().numpy()
    token = sup.token.cpu().numpy()
    prob = sup.prob.cpu().numpy()
    lse = sup.lse.cpu().numpy()
    n_compact = n_tie = 0
    for r in range(rows.shape[0]):
        ref_cut, rflags = W.warp_cutoff(rows[r], T, K, Pp)
        if rflags & O.FLAG_BAD_ROW:
            assert count[r] == 0 and gflags[r] & O.FLAG_BAD_ROW and np.isnan(lse[r])
            continue
        if (rflags | gflags[r]) & O.FLAG_NEAR_TIE:
            n_tie += 1
            continue
        vals = O.upcast(rows[r])
        y = vals / T
        keep = np.flatnonzero((vals >= ref_cut) & np.isfinite(vals))
        if count[r] < 0:
            # allowed only when the support does not fit, or top-p alone met a flat row
            few_finite = 0 < K < V and np.sort(vals)[-K] == -np.inf     # masked row: every entry is a candidate
            assert keep.size > cap or not (0 < K < V) or K > 512 or few_finite, (r, T, K, Pp, keep.size, cap)
            continue
        n_compact += 1
        # a kept entry whose mass exp((z - max) / T) underflows float64 has probability zero and is
        # not listed (the stated format of the support); right at the underflow either is accepted
        with np.errstate(under="ignore"):
            e_all = np.exp(y[keep] - y[keep].max())
        must = keep[e_all > 1e-300]
        listed = token[r, :count[r]]
        assert must.size <= count[r] <= keep.size, (r, T, K, Pp, count[r], must.size, keep.size)
        assert np.isin(must, listed).all() and np.isin(listed, keep).all(), (r, T, K, Pp)
        assert np.all(np.diff(listed) > 0), (r, T, K, Pp)
        on = np.isin(keep, listed)
        keep, e = keep[on], e_all[on]
        p_ref = e / e.sum()
        assert np.allclose(prob[r, :count[r]], p_ref, rtol=1e-12, atol=1e-300), (r, T, K, Pp)
        lse_ref = y[keep].max() + np.log(e.sum())
        assert abs(lse[r] - lse_ref) <= 1e-6 * max(1.0, abs(lse_ref)), (r, lse[r], lse_ref)
        # untouched beyond the count
        assert np.all(token[r, count[r]:] == -3) and np.all(prob[r, count[r]:] == -1.0)
    return n_compact, n_tie


@pytest.mark.parametrize("T,K,Pp,cap", [(0.7, 20, 0.8, 64), (0.95, 20, 0.6, 64), (0.6, 0, 0.9, 256),
                                        (1.0, 1, 1.0, 8), (1.0, 50, 1.0, 64), (0.5, 5, 0.999, 16),
                                        (1.0, 0, 1e-6, 4), (1.0, 0, 1.0, 1024), (1.0, 200, 1.0, 1024),
                                        (0.7, 20, 0.8, 4)])
def test_compact_supports_match_oracle(T, K, Pp, cap):
    T = _t32(T)
    compact = 0
    for idx, B, k, V, dtype in ((1, 3, 4, 32000, "bf16"), (3, 2, 3, 152064, "bf16"), (2, 2, 2, 20011, "bf16"),
                                (0, 2, 3, 4099, "f32"), (1, 2, 2, 9, "bf16"), (0, 1, 2, 1500, "f32")):
        cfg = svgen.make_config(idx, B=B, k=k, V=V, dtype=dtype)
        for name in ("z_t", "z_d"):
            c, _ = _check_supports(cfg[name], T, K, Pp, cap)
            compact += c
    if 0 < K <= 64 and cap >= 64:
        assert compact >= 40            # top-k rows always fit


def test_compact_bad_rows_and_masked_entries():
    z = torch.randn(6, 5000) * 3
    z[0, 7] = float("nan")
    z[1, :] = float("-inf")
    z[2, 11] = float("inf")
    z[3, 100:] = float("-inf")          # fewer finite entries than K
    z[4, ::2] = float("-inf")
    _check_supports(z, 1.0, 200, 0.95, 1024)
    _check_supports(z.to(torch.bfloat16), _t32(0.7), 20, 0.8, 64)


def test_compact_entries_whose_mass_underflows_are_not_listed():
    """A row whose largest entry stands hundreds of units above the rest at a low temperature:
    top-k keeps K entries, but all except the first have a mass below what float64 holds; the
    support lists the entries of positive probability only."""
    rng = np.random.default_rng(3)
    z = rng.standard_normal((4, 5000)).astype(np.float32)
    z[0, 17] = 300.0                       # (z - 300) / 0.3 < -745 for every other entry
    z[1, 4000] = 250.0
    z[1, 123] = 249.0                      # two entries with mass, eighteen without
    z[2] *= 300.0                          # a wide row: some of its top 20 underflow, some do not
    T = _t32(0.3)
    for dtype in (torch.float32, torch.bfloat16):
        t = torch.from_numpy(z).to(dtype)
        n_compact, _ = _check_supports(t, T, 20, 1.0, 64)
        assert n_compact == 4
        sup, _, _ = _compact(t.cuda(), T, 20, 1.0, 64)
        count = sup.count.cpu().numpy()
        assert count[0] == 1 and count[1] == 2 and 1 <= count[2] < 20 and count[3] == 20


def _supports_for(cfg_t, T, K, Pp, cap):
    sup, _, flags = _compact(cfg_t, T, K, Pp, cap)
    return sup, flags


def _outputs(B, k, with_kl=True):
    mk = lambda: torch.full((B, k), -7.0, dtype=torch.float32, device="cuda")
    return dict(lse_d=mk(), lse_c=mk(), S=mk(), A=mk(), KL=mk() if with_kl else None,
                H_d=mk() if with_kl else None, pd_x=mk(),
                flags=torch.full((B, k), 0xFFFF, dtype=torch.int32, device="cuda"))


def _redraw_tokens(y_d, seed):
    rng = np.random.default_rng(seed)
    B, k, V = y_d.shape
    x = np.zeros((B, k), dtype=np.int32)
    for b in range(B):
        for i in range(k):
            p = np.exp(y_d[b, i] - y_d[b, i].max())
            x[b, i] = rng.choice(V, p=p / p.sum())
    return x


CASES = [(1, 3, 4, 32000, "bf16"), (3, 2, 3, 152064, "bf16"), (0, 2, 3, 4099, "f32"), (2, 2, 3, 20011, "bf16")]


@pytest.mark.parametrize("pd_,pc_", [(SERIES[0], SERIES[0]), (SERIES[1], SERIES[2]), (SERIES[2], SERIES[1]),
                                     ((1.7, 3, 1.0), (0.4, 0, 0.5))])
def test_row_stats_sparse_matches_oracle(pd_, pc_):
    P = H.sv()
    checked = 0
    for idx, B, k, V, dtype in CASES:
        cfg = svgen.make_config(idx, seed=70 + idx, B=B, k=k, V=V, dtype=dtype, device="cuda")
        inp = H.oracle_inputs(cfg)
        Td, Tc = _t32(pd_[0]), _t32(pc_[0])
        y_d, _, f_d = W.warp_rows(inp["z_d"], Td, pd_[1], pd_[2])
        y_c, _, f_c = W.warp_rows(inp["z_c"], Tc, pc_[1], pc_[2])
        sup_d, gf_d = _supports_for(cfg["z_d"], Td, pd_[1], pd_[2], 256)
        sup_c, gf_c = _supports_for(cfg["z_c"], Tc, pc_[1], pc_[2], 256)
        for redraw in (False, True):
            x = _redraw_tokens(y_d, 5) if redraw else inp["x"]
            ref = O.row_stats(y_d, y_c, x)
            out = _outputs(B, k)
            P.sv_row_stats_sparse(sup_d, sup_c, H.dev(x, torch.int32), V, out["lse_d"], out["lse_c"], out["S"],
                                  out["A"], out["KL"], out["flags"], entropy_d=out["H_d"], pd_x=out["pd_x"])
            torch.cuda.synchronize()
            got = {n: t.cpu().numpy() for n, t in out.items()}
            # compare the pairs whose supports are compact and whose top-p decisions are not near ties
            skip = ((f_d | f_c | gf_d.reshape(B, k) | gf_c.reshape(B, k)) & O.FLAG_NEAR_TIE) != 0
            skip |= (got["flags"].astype(np.uint32) & NOT_COMPACT) != 0
            keep = ~skip
            checked += int(keep.sum())
            H.assert_row_stats({n: v[keep] for n, v in got.items()}, {n: np.asarray(v)[keep] for n, v in ref.items()})
    assert checked >= 30


@pytest.mark.parametrize("pt_,pd_", [(SERIES[0], SERIES[0]), (SERIES[1], SERIES[2]), (SERIES[2], SERIES[1]),
                                     ((0.5, 2, 1.0), (1.5, 0, 0.7))])
def test_verify_sample_sparse_matches_oracle(pt_, pd_):
    P = H.sv()
    checked = ties = 0
    for idx, B, k, V, dtype in CASES:
        cfg = svgen.make_config(idx, seed=170 + idx, B=B, k=k, V=V, dtype=dtype, device="cuda")
        inp = H.oracle_inputs(cfg)
        Tt, Td = _t32(pt_[0]), _t32(pd_[0])
        y_t, _, f_t = W.warp_rows(inp["z_t"], Tt, pt_[1], pt_[2])
        y_d, _, f_d = W.warp_rows(inp["z_d"], Td, pd_[1], pd_[2])
        sup_t, gf_t = _supports_for(cfg["z_t"], Tt, pt_[1], pt_[2], 256)
        sup_d, gf_d = _supports_for(cfg["z_d"], Td, pd_[1], pd_[2], 256)
        warp_tie = (((f_t | gf_t.reshape(B, k + 1)) & O.FLAG_NEAR_TIE) != 0).any(1) | \
                   (((f_d | gf_d.reshape(B, k)) & O.FLAG_NEAR_TIE) != 0).any(1)
        for redraw in (False, True):
            x = _redraw_tokens(y_d, 6) if redraw else inp["x"]
            for step in range(3):
                ref = H.oracle_verify(y_t, y_d, x, seed=77, step=step)
                tokens = torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda")
                n_acc = torch.full((B,), -5, dtype=torch.int32, device="cuda")
                flags = torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda")
                ratio = torch.full((B, k), -5.0, dtype=torch.float32, device="cuda")
                P.sv_verify_sample_sparse(sup_t, None, sup_d, H.dev(x, torch.int32), None, V, 77, step, tokens,
                                          n_acc, flags, ratio)
                torch.cuda.synchronize()
                got = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
                           flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
                keep = ~warp_tie & ((got["flags"] & NOT_COMPACT) == 0)
                sub = lambda d: {n: ([v[i] for i in np.flatnonzero(keep)] if isinstance(v, list)
                                     else np.asarray(v)[keep]) for n, v in d.items()}
                t, _ = H.assert_verify(sub(got), sub(ref), k)
                ties += t
                checked += int(keep.sum())
    assert checked >= 15 and ties <= max(1, checked // 20)     # flat top-p-only rows are not compact


def test_verify_sample_sparse_packed_ragged_and_gamma():
    P = H.sv()
    B, k, V = 5, 4, 32000
    cfg = svgen.make_config(1, seed=411, B=B, k=k, V=V, dtype="bf16", device="cuda")
    inp = H.oracle_inputs(cfg)
    T, K, Pp = _t32(0.7), 20, 0.8
    gamma = np.array([0, 4, 2, 1, 3], dtype=np.int32)
    offs = np.concatenate([[0], np.cumsum(gamma + 1)]).astype(np.int32)
    packed = np.concatenate([inp["z_t"][b, :gamma[b] + 1] for b in range(B)], axis=0)
    z_t_packed = torch.cat([cfg["z_t"][b, :gamma[b] + 1] for b in range(B)], dim=0).contiguous()
    y_tp, _, f_t = W.warp_rows(packed, T, K, Pp)
    y_d, _, f_d = W.warp_rows(inp["z_d"], T, K, Pp)
    assert not ((f_t | 0) & O.FLAG_NEAR_TIE).any() and not (f_d & O.FLAG_NEAR_TIE).any()
    x = _redraw_tokens(y_d, 7)
    sup_t, _ = _supports_for(z_t_packed, T, K, Pp, 64)
    sup_d, _ = _supports_for(cfg["z_d"], T, K, Pp, 64)
    ref = H.oracle_verify(y_tp, y_d, x, gamma=gamma, t_offsets=offs, seed=5, step=9)
    tokens = torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda")
    n_acc = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    flags = torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda")
    ratio = torch.full((B, k), -5.0, dtype=torch.float32, device="cuda")
    P.sv_verify_sample_sparse(sup_t, H.dev(offs, torch.int32), sup_d, H.dev(x, torch.int32),
                              H.dev(gamma, torch.int32), V, 5, 9, tokens, n_acc, flags, ratio)
    torch.cuda.synchronize()
    got = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
               flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
    H.assert_verify(got, ref, k)


def test_sparse_flags_rows_without_compact_support_and_bad_rows():
    P = H.sv()
    B, k, V = 2, 3, 5000
    cfg = svgen.make_config(0, seed=45, B=B, k=k, V=V, dtype="f32", device="cuda")
    z_d = cfg["z_d"].clone()
    z_d[1, 2, 5] = float("nan")
    T = _t32(0.8)
    sup_d, _ = _supports_for(z_d, T, 20, 1.0, 8)            # top-k 20 does not fit 8 entries
    sup_c, _ = _supports_for(cfg["z_c"], T, 5, 1.0, 8)
    count = sup_d.count.cpu().numpy()
    assert (count[:5] == -1).all() and count[5] == 0
    out = _outputs(B, k)
    P.sv_row_stats_sparse(sup_d, sup_c, cfg["x"], V, out["lse_d"], out["lse_c"], out["S"], out["A"], out["KL"],
                          out["flags"], entropy_d=out["H_d"], pd_x=out["pd_x"])
    torch.cuda.synchronize()
    fl = out["flags"].cpu().numpy().reshape(-1).astype(np.uint32)
    assert (fl[:5] == NOT_COMPACT).all() and fl[5] == O.FLAG_BAD_ROW
    assert np.isnan(out["S"].cpu().numpy()).all()
    sup_t, _ = _supports_for(cfg["z_t"], T, 5, 1.0, 8)
    tokens = torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda")
    n_acc = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    flags = torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda")
    P.sv_verify_sample_sparse(sup_t, None, sup_d, cfg["x"], None, V, 1, 0, tokens, n_acc, flags)
    torch.cuda.synchronize()
    fl = flags.cpu().numpy().astype(np.uint32)
    assert (fl & NOT_COMPACT).all() and (fl & O.FLAG_BAD_ROW).all()
    assert (n_acc.cpu().numpy() == 0).all()                 # a row without support rejects there


def test_sparse_step_end_to_end_against_dense_warped_path():
    """Whole warped step on compacted supports vs the dense warped entry points on
    the same inputs (both already checked against the oracle): identical lengths,
    accept counts and tokens; statistics equal to rounding."""
    P = H.sv()
    idx, B, k, V = 3, 16, 8, 152064
    cfg = svgen.make_config(idx, seed=2025, B=B, k=k, V=V, dtype="bf16", device="cuda")
    T, K, Pp, cap = _t32(0.7), 20, 0.8, 64
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    cut_t, cut_d, cut_c = f32(B * (k + 1)), f32(B * k), f32(B * k)
    wf = [i32(B * (k + 1)), i32(B * k), i32(B * k)]
    sup_t, sup_d, sup_c = P.Supports(B * (k + 1), cap), P.Supports(B * k, cap), P.Supports(B * k, cap)
    P.sv_warp_compact(cfg["z_t"], T, K, Pp, sup_t, cut_t, wf[0])
    P.sv_warp_compact(cfg["z_d"], T, K, Pp, sup_d, cut_d, wf[1])
    P.sv_warp_compact(cfg["z_c"], T, K, Pp, sup_c, cut_c, wf[2])
    assert (sup_t.count.cpu().numpy() > 0).all() and (sup_d.count.cpu().numpy() > 0).all()
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = H.dev(svgen.latency_table(B * k), torch.float32)
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    res = {}
    for mode in ("dense", "sparse"):
        lse_d, lse_c, S, A, p_hat = (f32(B, k) for _ in range(5))
        gamma, offs, total = i32(B), i32(B + 1), i32(1)
        tokens, n_acc, flags, ratio = i32(B, k + 1), i32(B), i32(B), f32(B, k)
        if mode == "dense":
            P.sv_row_stats_warped(cfg["z_d"], cfg["z_c"], cfg["x"], T, cut_d, T, cut_c, lse_d, lse_c, S, A, None,
                                  None, ws)
        else:
            P.sv_row_stats_sparse(sup_d, sup_c, cfg["x"], V, lse_d, lse_c, S, A)
        P.sv_accept_estimate(S, A, H.dev(edges_s), H.dev(edges_a), H.dev(table), p_hat, None)
        P.sv_select_length(p_hat, lat, P.SV_BATCH_GREEDY, gamma, offs, total)
        if mode == "dense":
            P.sv_verify_sample_warped(cfg["z_t"], None, cfg["z_d"], cfg["x"], gamma, T, cut_t, T, cut_d, 11, 4,
                                      tokens, n_acc, flags, ratio, ws)
        else:
            P.sv_verify_sample_sparse(sup_t, None, sup_d, cfg["x"], gamma, V, 11, 4, tokens, n_acc, flags, ratio)
        torch.cuda.synchronize()
        res[mode] = {n: t.cpu().numpy() for n, t in dict(S=S, A=A, lse_d=lse_d, gamma=gamma, tokens=tokens,
                                                         n_acc=n_acc, flags=flags, ratio=ratio).items()}
    d, s = res["dense"], res["sparse"]
    assert H.close(d["S"], s["S"], 2e-6, 1e-7).all() and H.close(d["A"], s["A"], 2e-6, 1e-30).all()
    assert H.close(d["lse_d"], s["lse_d"], 2e-6, 1e-6).all()
    near = (d["flags"] | s["flags"]) & (O.FLAG_NEAR_TIE | O.FLAG_NEAR_CDF_EDGE)
    if np.array_equal(d["gamma"], s["gamma"]):              # (a bin edge within rounding of S or A could differ)
        ok = near == 0
        assert np.array_equal(d["n_acc"][ok], s["n_acc"][ok])
        assert np.array_equal(d["tokens"][ok], s["tokens"][ok])
    else:
        pytest.skip("estimates fell on different sides of a bin edge")


def test_accept_ratio_sparse_matches_oracle():
    """X = P_t(x) / P_d(x) of every drafted position under the warped distributions
    (profile construction), against the oracle's ratio on warped rows."""
    from oracle import profile_oracle as PO
    P = H.sv()
    for (idx, B, k, V, dtype), (T, K, Pp) in zip(CASES, SERIES + [(1.3, 50, 0.95)]):
        T = _t32(T)
        cfg = svgen.make_config(idx, seed=270 + idx, B=B, k=k, V=V, dtype=dtype, device="cuda")
        inp = H.oracle_inputs(cfg)
        y_t, _, f_t = W.warp_rows(inp["z_t"], T, K, Pp)
        y_d, _, f_d = W.warp_rows(inp["z_d"], T, K, Pp)
        sup_t, gf_t = _supports_for(cfg["z_t"], T, K, Pp, 256)
        sup_d, gf_d = _supports_for(cfg["z_d"], T, K, Pp, 256)
        for redraw in (False, True):
            x = _redraw_tokens(y_d, 11) if redraw else inp["x"]
            ref, _ = PO.accept_probability_ratio(y_t, y_d, x)
            ratio = torch.full((B, k), -5.0, dtype=torch.float32, device="cuda")
            flags = torch.full((B, k), 77, dtype=torch.int32, device="cuda")
            P.sv_accept_ratio_sparse(sup_t, sup_d, H.dev(x, torch.int32), V, ratio, flags)
            torch.cuda.synchronize()
            got, fl = ratio.cpu().numpy(), flags.cpu().numpy().astype(np.uint32)
            tie = ((f_t[:, :k] | f_d | gf_t.reshape(B, k + 1)[:, :k] | gf_d.reshape(B, k)) & O.FLAG_NEAR_TIE) != 0
            ok = ~tie & (fl == 0)
            assert ok.sum() >= B * k // 2
            assert H.close(got[ok], np.asarray(ref)[ok], H.REL, 1e-30).all(), (got[ok], np.asarray(ref)[ok])


def _mixed_rows(rows, V, seed):
    """Rows of every kind in turn, so that all paths of the kernel run side by side in one
    launch: peaked, nearly flat, masked, bad, tied, empty."""
    rng = np.random.default_rng(seed)
    z = (3.0 * rng.standard_normal((rows, V))).astype(np.float32)
    kind = np.arange(rows) % 7
    z[kind == 1] *= 0.003                                         # nearly flat
    for r in np.flatnonzero(kind == 2):
        z[r, rng.random(V) < 0.995] = -np.inf                     # a handful of finite entries
    for r in np.flatnonzero(kind == 3):
        z[r, rng.integers(V)] = np.nan if r % 2 else np.inf       # bad rows
    z[kind == 4] = np.round(z[kind == 4] * 2) / 2                 # ties
    z[kind == 5] = -np.inf                                        # nothing finite: bad as well
    return torch.from_numpy(z)


@pytest.mark.parametrize("V,dtype", [(4104, torch.bfloat16), (4100, torch.float32), (4101, torch.bfloat16)])
def test_launches_with_more_rows_than_resident_workgroups(V, dtype):
    """A launch of more rows than the chip holds workgroups at once (1024), with rows of every
    kind mixed: every row against the oracle, and bit for bit what launches of at most 1000
    rows give (a row's result must not depend on what else the launch holds)."""
    P = H.sv()
    rows = 2 * 1024 + 517
    z = _mixed_rows(rows, V, seed=V).to(dtype)
    zc = z.cuda()
    for T, K, Pp, cap in ((0.7, 20, 0.8, 64), (0.6, 0, 0.9, 256), (1.0, 0, 1.0, 64)):
        T = _t32(T)
        n_compact, _ = _check_supports(z, T, K, Pp, cap)
        if K:
            assert n_compact > rows // 2
        whole, cut_w, flags_w = _compact(zc, T, K, Pp, cap)
        for r0 in range(0, rows, 1000):
            part, cut_p, flags_p = _compact(zc[r0:r0 + 1000], T, K, Pp, cap)
            n = part.count.shape[0]
            assert torch.equal(part.count, whole.count[r0:r0 + n])
            assert torch.equal(part.token, whole.token[r0:r0 + n])
            assert torch.equal(part.prob.view(torch.int64), whole.prob[r0:r0 + n].view(torch.int64))
            assert torch.equal(part.lse.view(torch.int32), whole.lse[r0:r0 + n].view(torch.int32))
            assert np.array_equal(cut_p.view(np.uint32), cut_w[r0:r0 + n].view(np.uint32))
            assert np.array_equal(flags_p, flags_w[r0:r0 + n])
