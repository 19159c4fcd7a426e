"""GPU parity of the warped entry points (temperature, top-k, top-p applied to
the draft, companion and target distributions) against the oracle: the oracle
warps the rows first (oracle/warp_oracle.warp_rows: z / T with the dropped
entries at -inf) and then runs the ordinary row_stats / verify_sample on them.
Temperatures are float32 values on both sides."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O
from oracle import warp_oracle as W

import harness as H

pytestmark = pytest.mark.gpu

# (temperature, top_k, top_p) as in the paper's appendix table of sampling hyper-parameters
SERIES = [(0.7, 20, 0.8), (0.95, 20, 0.6), (0.6, 0, 0.9)]


def _t32(T):
    return float(np.float32(T))


def _cut32(cut):
    """Oracle cutoffs (values of the row, -inf or NaN) as a float32 device tensor."""
    return H.dev(np.asarray(cut, dtype=np.float32))


def _gpu_row_stats_warped(z_d, z_c, x, Td, cut_d, Tc, cut_c, with_kl=True):
    P = H.sv()
    B, k, V = z_d.shape
    mk = lambda: torch.full((B, k), -7.0, dtype=torch.float32, device="cuda")
    out = dict(lse_d=mk(), lse_c=mk(), S=mk(), A=mk(), KL=mk() if with_kl else None,
               H_d=mk() if with_kl else None, pd_x=mk(),
               flags=torch.full((B, k), 0xFFFF, dtype=torch.int32, device="cuda"))
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(z_d))
    P.sv_row_stats_warped(z_d, z_c, x, Td, cut_d, Tc, cut_c, out["lse_d"], out["lse_c"], out["S"], out["A"],
                          out["KL"], out["flags"], ws, entropy_d=out["H_d"], pd_x=out["pd_x"])
    torch.cuda.synchronize()
    return {n: (None if t is None else t.cpu().numpy()) for n, t in out.items()}


def _gpu_verify_warped(z_t, z_d, x, Tt, cut_t, Td, cut_d, gamma=None, t_offsets=None, seed=0, step=0):
    P = H.sv()
    B, k, V = z_d.shape
    tokens = torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda")
    n_acc = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    flags = torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda")
    ratio = torch.full((B, k), -5.0, dtype=torch.float32, device="cuda")
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(z_d))
    g = None if gamma is None else H.dev(gamma, torch.int32)
    o = None if t_offsets is None else H.dev(t_offsets, torch.int32)
    P.sv_verify_sample_warped(z_t, o, z_d, x, g, Tt, cut_t, Td, cut_d, seed, step, tokens, n_acc, flags, ratio, ws)
    torch.cuda.synchronize()
    return dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
                flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())


def _redraw_tokens(y_d, seed):
    """Drafted tokens drawn from the warped draft distribution (as a real run would)."""
    rng = np.random.default_rng(seed)
    B, k, V = y_d.shape
    x = np.zeros((B, k), dtype=np.int32)
    for b in range(B):
        for i in range(k):
            row = y_d[b, i]
            p = np.exp(row - row.max())
            x[b, i] = rng.choice(V, p=p / p.sum())
    return x


CASES = [(1, 3, 4, 32000, "bf16"), (3, 2, 3, 152064, "bf16"), (0, 2, 3, 4099, "f32"), (2, 2, 3, 20011, "bf16")]


@pytest.mark.parametrize("pd_,pc_", [(SERIES[0], SERIES[0]), (SERIES[1], SERIES[2]), (SERIES[2], (1.0, 0, 1.0)),
                                     ((1.0, 0, 1.0), (1.0, 0, 1.0)), ((1.7, 3, 1.0), (0.4, 0, 0.5))])
def test_row_stats_warped_matches_oracle(pd_, pc_):
    for idx, B, k, V, dtype in CASES:
        cfg = svgen.make_config(idx, seed=90 + idx, B=B, k=k, V=V, dtype=dtype, device="cuda")
        inp = H.oracle_inputs(cfg)
        Td, Tc = _t32(pd_[0]), _t32(pc_[0])
        y_d, cut_d, _ = W.warp_rows(inp["z_d"], Td, pd_[1], pd_[2])
        y_c, cut_c, _ = W.warp_rows(inp["z_c"], Tc, pc_[1], pc_[2])
        for redraw in (False, True):
            x = _redraw_tokens(y_d, 5) if redraw else inp["x"]
            ref = O.row_stats(y_d, y_c, x)
            got = _gpu_row_stats_warped(cfg["z_d"], cfg["z_c"], H.dev(x, torch.int32), Td, _cut32(cut_d),
                                        Tc, _cut32(cut_c))
            H.assert_row_stats(got, ref)
            got = _gpu_row_stats_warped(cfg["z_d"], cfg["z_c"], H.dev(x, torch.int32), Td, _cut32(cut_d),
                                        Tc, _cut32(cut_c), with_kl=False)
            H.assert_row_stats(got, ref, with_kl=False)


@pytest.mark.parametrize("pt_,pd_", [(SERIES[0], SERIES[0]), (SERIES[1], SERIES[2]), (SERIES[2], SERIES[1]),
                                     ((1.0, 0, 1.0), (1.0, 0, 1.0)), ((0.5, 2, 1.0), (1.5, 0, 0.7))])
def test_verify_sample_warped_matches_oracle(pt_, pd_):
    ties = edges = total = 0
    for idx, B, k, V, dtype in CASES:
        cfg = svgen.make_config(idx, seed=190 + idx, B=B, k=k, V=V, dtype=dtype, device="cuda")
        inp = H.oracle_inputs(cfg)
        Tt, Td = _t32(pt_[0]), _t32(pd_[0])
        y_t, cut_t, _ = W.warp_rows(inp["z_t"], Tt, pt_[1], pt_[2])
        y_d, cut_d, _ = W.warp_rows(inp["z_d"], Td, pd_[1], pd_[2])
        for redraw in (False, True):
            x = _redraw_tokens(y_d, 6) if redraw else inp["x"]
            for step in range(3):
                ref = H.oracle_verify(y_t, y_d, x, seed=77, step=step)
                got = _gpu_verify_warped(cfg["z_t"], cfg["z_d"], H.dev(x, torch.int32), Tt, _cut32(cut_t),
                                         Td, _cut32(cut_d), seed=77, step=step)
                t, e = H.assert_verify(got, ref, k)
                ties, edges, total = ties + t, edges + e, total + B
    assert ties <= max(1, total // 20), (ties, total)


def test_verify_sample_warped_packed_and_ragged():
    B, k, V = 5, 4, 32000
    cfg = svgen.make_config(1, seed=311, B=B, k=k, V=V, dtype="bf16", device="cuda")
    inp = H.oracle_inputs(cfg)
    T, K, Pp = _t32(0.7), 20, 0.8
    gamma = np.array([0, 4, 2, 1, 3], dtype=np.int32)
    offs = np.concatenate([[0], np.cumsum(gamma + 1)]).astype(np.int32)
    packed = np.concatenate([inp["z_t"][b, :gamma[b] + 1] for b in range(B)], axis=0)
    z_t_packed = torch.cat([cfg["z_t"][b, :gamma[b] + 1] for b in range(B)], dim=0).contiguous()
    y_tp, cut_tp, _ = W.warp_rows(packed, T, K, Pp)
    y_d, cut_d, _ = W.warp_rows(inp["z_d"], T, K, Pp)
    x = _redraw_tokens(y_d, 7)
    ref = H.oracle_verify(y_tp, y_d, x, gamma=gamma, t_offsets=offs, seed=5, step=9)
    got = _gpu_verify_warped(z_t_packed, cfg["z_d"], H.dev(x, torch.int32), T, _cut32(cut_tp), T, _cut32(cut_d),
                             gamma=gamma, t_offsets=offs, seed=5, step=9)
    H.assert_verify(got, ref, k)


def test_unit_warp_equals_plain_entry_points():
    """T = 1 without cutoffs: sv_verify_sample_warped runs the same kernels as
    sv_verify_sample and must give identical bits; sv_row_stats_warped runs the
    plain two-sweep kernel and must agree to rounding."""
    cfg = svgen.make_config(1, seed=12, B=4, k=4, V=32000, dtype="bf16", device="cuda")
    plain = H.gpu_verify(cfg["z_t"], cfg["z_d"], cfg["x"], seed=3, step=1)
    warped = _gpu_verify_warped(cfg["z_t"], cfg["z_d"], cfg["x"], 1.0, None, 1.0, None, seed=3, step=1)
    for name in ("tokens", "n_accept", "flags"):
        assert np.array_equal(plain[name], warped[name]), name
    assert np.array_equal(plain["ratio"], warped["ratio"], equal_nan=True)
    a = H.gpu_row_stats(cfg["z_d"], cfg["z_c"], cfg["x"])
    b = _gpu_row_stats_warped(cfg["z_d"], cfg["z_c"], cfg["x"], 1.0, None, 1.0, None)
    for name in ("lse_d", "lse_c", "S", "A", "KL", "H_d", "pd_x"):
        assert H.close(b[name], a[name], 2e-6, 1e-7).all(), name


def test_warped_bad_rows_masked_entries_and_tokens_outside_support():
    B, k, V = 3, 3, 5000
    cfg = svgen.make_config(0, seed=44, B=B, k=k, V=V, dtype="f32", device="cuda")
    z_d, z_c, z_t = cfg["z_d"].clone(), cfg["z_c"].clone(), cfg["z_t"].clone()
    z_d[0, 1, 17] = float("nan")                  # bad draft row
    z_c[1, 0, :] = float("-inf")                  # companion row without a finite entry
    z_t[2, 1, 100:4000] = float("-inf")           # masked vocabulary range in a target row
    x = cfg["x"].clone()
    x[2, 0] = int(torch.argmin(z_d[2, 0]))        # a token the draft's top-k certainly drops
    zn = dict(z_t=z_t.cpu().numpy(), z_d=z_d.cpu().numpy(), z_c=z_c.cpu().numpy(), x=x.cpu().numpy())
    T, K, Pp = _t32(0.8), 50, 0.95
    y_t, cut_t, _ = W.warp_rows(zn["z_t"], T, K, Pp)
    y_d, cut_d, _ = W.warp_rows(zn["z_d"], T, K, Pp)
    y_c, cut_c, _ = W.warp_rows(zn["z_c"], T, K, Pp)
    ref = O.row_stats(y_d, y_c, zn["x"])
    got = _gpu_row_stats_warped(z_d, z_c, x, T, _cut32(cut_d), T, _cut32(cut_c))
    H.assert_row_stats(got, ref)
    assert got["flags"][0, 1] & O.FLAG_BAD_ROW and got["flags"][1, 0] & O.FLAG_BAD_ROW
    assert got["A"][2, 0] == 1.0 and got["pd_x"][2, 0] == 0.0
    ref = H.oracle_verify(y_t, y_d, zn["x"], seed=1, step=2)
    got = _gpu_verify_warped(z_t, z_d, x, T, _cut32(cut_t), T, _cut32(cut_d), seed=1, step=2)
    H.assert_verify(got, ref, k)


def test_decode_step_with_gpu_cutoffs_end_to_end():
    """The whole warped step on the GPU - cutoffs, indicators, estimate, lengths,
    verification - against the oracle chain.  Sequences with a row whose top-p
    decision either side flags as a near tie are counted and skipped."""
    P = H.sv()
    idx, B, k, V = 3, 6, 4, 152064
    cfg = svgen.make_config(idx, seed=2024, B=B, k=k, V=V, dtype="bf16", device="cuda")
    inp = H.oracle_inputs(cfg)
    (Tt, Kt, Pt), (Td, Kd, Pd), (Tc, Kc, Pc) = [(_t32(a), b, c) for a, b, c in
                                                 (SERIES[0], SERIES[0], SERIES[2])]
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    cut_t, cut_d, cut_c = f32(B * (k + 1)), f32(B * k), f32(B * k)
    wf_t, wf_d, wf_c = i32(B * (k + 1)), i32(B * k), i32(B * k)
    P.sv_warp_cutoffs(cfg["z_t"], Tt, Kt, Pt, cut_t, wf_t)
    P.sv_warp_cutoffs(cfg["z_d"], Td, Kd, Pd, cut_d, wf_d)
    P.sv_warp_cutoffs(cfg["z_c"], Tc, Kc, Pc, cut_c, wf_c)
    y_t, rcut_t, rf_t = W.warp_rows(inp["z_t"], Tt, Kt, Pt)
    y_d, rcut_d, rf_d = W.warp_rows(inp["z_d"], Td, Kd, Pd)
    y_c, rcut_c, rf_c = W.warp_rows(inp["z_c"], Tc, Kc, Pc)
    x = _redraw_tokens(y_d, 8)
    xg = H.dev(x, torch.int32)
    tie = ((wf_t.cpu().numpy().reshape(B, k + 1) | rf_t) & O.FLAG_NEAR_TIE).any(1) | \
          ((wf_d.cpu().numpy().reshape(B, k) | rf_d) & O.FLAG_NEAR_TIE).any(1) | \
          ((wf_c.cpu().numpy().reshape(B, k) | rf_c) & O.FLAG_NEAR_TIE).any(1)
    keep = ~tie
    assert keep.sum() >= B - 2, tie
    # the GPU cutoffs select the same kept sets as the oracle's on the compared sequences
    for name, gc, rc, z in (("t", cut_t, rcut_t, inp["z_t"]), ("d", cut_d, rcut_d, inp["z_d"]),
                            ("c", cut_c, rcut_c, inp["z_c"])):
        g = gc.cpu().numpy().reshape(rc.shape)
        vals = O.upcast(z)
        same = ((vals >= g[..., None]) == (vals >= rc[..., None])).all(-1).all(-1)
        assert same[keep].all(), name

    edges_s, edges_a, table = svgen.profile_table(10, 10)
    latency = svgen.latency_table(B * k)
    lse_d, lse_c, S, A, p_hat = (f32(B, k) for _ in range(5))
    gamma, offs, total = i32(B), i32(B + 1), i32(1)
    tokens, n_acc, flags, ratio = i32(B, k + 1), i32(B), i32(B), f32(B, k)
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    P.sv_row_stats_warped(cfg["z_d"], cfg["z_c"], xg, Td, cut_d, Tc, cut_c, lse_d, lse_c, S, A, None, None, ws)
    P.sv_accept_estimate(S, A, H.dev(edges_s), H.dev(edges_a), H.dev(table), p_hat, None)
    P.sv_select_length(p_hat, H.dev(latency, torch.float32), P.SV_BATCH_GREEDY, gamma, offs, total)
    P.sv_verify_sample_warped(cfg["z_t"], None, cfg["z_d"], xg, gamma, Tt, cut_t, Td, cut_d, 11, 4, tokens, n_acc,
                              flags, ratio, ws)
    torch.cuda.synchronize()

    r = O.row_stats(y_d, y_c, x)
    assert H.close(S.cpu().numpy()[keep], r["S"][keep], H.REL).all()
    assert H.close(A.cpu().numpy()[keep], r["A"][keep], H.REL, 1e-30).all()
    # lengths and verification from the GPU's own float32 S, A (the oracle's rule on the same inputs)
    p_ref, near = O.accept_estimate(S.cpu().numpy(), A.cpu().numpy(), edges_s, edges_a, table)
    assert np.array_equal(p_hat.cpu().numpy(), p_ref)
    sel = O.select_length(p_ref, latency, O.MODE_BATCH_GREEDY)
    g_ref = sel[0] if isinstance(sel, tuple) else sel["gamma"]
    assert np.array_equal(gamma.cpu().numpy(), g_ref)
    ref = H.oracle_verify(y_t, y_d, x, gamma=g_ref, seed=11, step=4)
    got = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
               flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
    sub = lambda d: {n: ([v[i] for i in np.flatnonzero(keep)] if isinstance(v, list) else np.asarray(v)[keep])
                     for n, v in d.items()}
    H.assert_verify(sub(got), sub(ref), k)


@pytest.mark.parametrize("T", [0.01, 0.05, 20.0, 100.0])
def test_extreme_temperatures(T):
    """Very sharp and very flat warped distributions, dense and compacted."""
    P = H.sv()
    T = _t32(T)
    K, Pp = (0, 1.0) if T > 1 else (50, 0.99)
    for idx, B, k, V, dtype in ((1, 2, 3, 32000, "bf16"), (0, 2, 2, 4099, "f32")):
        cfg = svgen.make_config(idx, seed=600 + idx, B=B, k=k, V=V, dtype=dtype, device="cuda")
        inp = H.oracle_inputs(cfg)
        y_t, cut_t, f_t = W.warp_rows(inp["z_t"], T, K, Pp)
        y_d, cut_d, f_d = W.warp_rows(inp["z_d"], T, K, Pp)
        y_c, cut_c, f_c = W.warp_rows(inp["z_c"], T, K, Pp)
        x = _redraw_tokens(y_d, 9)
        xg = H.dev(x, torch.int32)
        pair_ok = ((f_d | f_c) & O.FLAG_NEAR_TIE) == 0
        ref = O.row_stats(y_d, y_c, x)
        got = _gpu_row_stats_warped(cfg["z_d"], cfg["z_c"], xg, T, _cut32(cut_d), T, _cut32(cut_c))
        H.assert_row_stats({n: v[pair_ok] for n, v in got.items()}, {n: np.asarray(v)[pair_ok] for n, v in ref.items()})
        vref = H.oracle_verify(y_t, y_d, x, seed=3, step=8)
        vgot = _gpu_verify_warped(cfg["z_t"], cfg["z_d"], xg, T, _cut32(cut_t), T, _cut32(cut_d), seed=3, step=8)
        seq_ok = ~(((f_t & O.FLAG_NEAR_TIE) != 0).any(1) | ((f_d & O.FLAG_NEAR_TIE) != 0).any(1))
        sub = lambda d: {n: ([v[i] for i in np.flatnonzero(seq_ok)] if isinstance(v, list) else np.asarray(v)[seq_ok])
                         for n, v in d.items()}
        H.assert_verify(sub(vgot), sub(vref), k)
        if T < 1:                                        # sharp rows compact to a handful of tokens
            sup_d = P.Supports(B * k, 64)
            gf = torch.zeros(B * k, dtype=torch.int32, device="cuda")
            P.sv_warp_compact(cfg["z_d"], T, K, Pp, sup_d, None, gf)
            torch.cuda.synchronize()
            count = sup_d.count.cpu().numpy().reshape(B, k)
            tok = sup_d.token.cpu().numpy().reshape(B, k, -1)
            prob = sup_d.prob.cpu().numpy().reshape(B, k, -1)
            gfn = gf.cpu().numpy().reshape(B, k).astype(np.uint32)
            for b in range(B):
                for i in range(k):
                    if (gfn[b, i] | f_d[b, i]) & O.FLAG_NEAR_TIE or count[b, i] < 0:
                        continue
                    keep = np.flatnonzero(np.isfinite(y_d[b, i]) & (np.exp(y_d[b, i] - y_d[b, i].max()) > 0))
                    assert np.array_equal(tok[b, i, :count[b, i]], keep)
                    e = np.exp(y_d[b, i][keep] - y_d[b, i].max())
                    assert np.allclose(prob[b, i, :count[b, i]], e / e.sum(), rtol=1e-12, atol=0)


@pytest.mark.parametrize("T,K,Pp", SERIES)
@pytest.mark.parametrize("t_rows", ["k", "k+1"])
def test_accept_ratio_warped_every_position(T, K, Pp, t_rows):
    """X = P_t(x) / P_d(x) of every drafted position under the warped distributions, on the
    logits themselves (profiles for rows that do not compact), against the oracle's ratio on
    warped rows; drafted tokens both from the unwarped and from the warped draft distribution,
    with the oracle's own cutoffs and with those of sv_warp_cutoffs."""
    from oracle import profile_oracle as PO
    P = H.sv()
    T = _t32(T)
    B, k, V = 5, 4, 30000
    cfg = svgen.make_config(3, seed=640, B=B, k=k, V=V, dtype="bf16", device="cuda")
    z_t = cfg["z_t"] if t_rows == "k+1" else cfg["z_t"][:, :k].contiguous()
    inp = H.oracle_inputs(cfg)
    y_t, c_t, f_t = W.warp_rows(svgen.to_numpy_bits(z_t), T, K, Pp)
    y_d, c_d, f_d = W.warp_rows(inp["z_d"], T, K, Pp)
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    rng = np.random.default_rng(3)
    x_warped = inp["x"].copy()
    for b in range(B):                     # a token of the warped draft's support for half of the positions
        for i in range(0, k, 2):
            x_warped[b, i] = rng.choice(np.nonzero(np.isfinite(y_d[b, i]))[0])
    gcut_t = torch.empty(z_t.shape[0] * z_t.shape[1], dtype=torch.float32, device="cuda")
    gcut_d = torch.empty(B * k, dtype=torch.float32, device="cuda")
    gf_t, gf_d = torch.zeros_like(gcut_t, dtype=torch.int32), torch.zeros_like(gcut_d, dtype=torch.int32)
    P.sv_warp_cutoffs(z_t, T, K, Pp, gcut_t, gf_t)
    P.sv_warp_cutoffs(cfg["z_d"], T, K, Pp, gcut_d, gf_d)
    checked = 0
    for x in (inp["x"], x_warped):
        ref, _ = PO.accept_probability_ratio(y_t, y_d, x)
        for cuts in ((_cut32(c_t), _cut32(c_d)), (gcut_t, gcut_d)):
            ratio = torch.full((B, k), -5.0, dtype=torch.float32, device="cuda")
            flags = torch.full((B, k), 77, dtype=torch.int32, device="cuda")
            P.sv_accept_ratio_warped(z_t, cfg["z_d"], H.dev(x, torch.int32), T, cuts[0], T, cuts[1], ratio, flags, ws)
            torch.cuda.synchronize()
            got, fl = ratio.cpu().numpy(), flags.cpu().numpy()
            tie = ((f_t[:, :k] | f_d | gf_t.cpu().numpy().reshape(B, -1)[:, :k].astype(np.uint32)
                    | gf_d.cpu().numpy().reshape(B, k).astype(np.uint32)) & O.FLAG_NEAR_TIE) != 0
            assert (fl == 0).all()
            ok = ~tie
            assert H.close(got[ok], np.asarray(ref)[ok], H.REL, 1e-30).all(), (got[ok], np.asarray(ref)[ok])
            checked += int(ok.sum())
    assert checked >= 3 * B * k
