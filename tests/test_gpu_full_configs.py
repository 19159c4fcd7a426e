"""GPU parity at the full sizes of the five workload configurations, in the
launch configuration bench.py times, on every output (the oracle finishes each
config in well under a minute).  Config 5 runs the whole chain with the ragged
layout: lengths from sv_select_length, target rows packed for the selected
positions plus the bonus row, int32 offsets."""
import time

import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu


def _stage_isolated(index):
    t0 = time.time()
    cfg = svgen.make_config(index)
    d = {n: cfg[n].cuda() for n in ("z_t", "z_d", "z_c", "x")}
    oi = H.oracle_inputs(cfg)
    B, k = cfg["B"], cfg["k"]
    print(f"\n[{cfg['name']}] generated in {time.time() - t0:.1f}s", flush=True)

    t0 = time.time()
    ref = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
    got = H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl=True)
    H.assert_row_stats(got, ref, True)
    got = H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl=False)
    H.assert_row_stats(got, ref, False)
    print(f"  row_stats ok ({time.time() - t0:.1f}s)", flush=True)

    edges_s, edges_a, table = svgen.profile_table(10, 10)
    S32, A32 = ref["S"].astype(np.float32), ref["A"].astype(np.float32)
    rp, rflag = O.accept_estimate(S32, A32, edges_s, edges_a, table)
    gp, gflag = H.gpu_accept_estimate(S32, A32, edges_s, edges_a, table)
    assert np.array_equal(gp, rp) and np.array_equal(gflag, rflag)

    lat = svgen.latency_table(B * k)
    for mode, l in ((O.MODE_BATCH_GREEDY, lat), (O.MODE_PER_SEQUENCE, lat[:k + 1])):
        rg, ro, rm = O.select_length(rp, l, mode)
        gg, go, gm = H.gpu_select_length(rp, l, mode)
        assert gm == rm and np.array_equal(gg, rg) and np.array_equal(go, ro)
    print("  accept_estimate / select_length ok", flush=True)
    return cfg, d, oi, rp, lat


@pytest.mark.parametrize("index", [2, 3])
def test_full_config_dense(index):
    cfg, d, oi, rp, lat = _stage_isolated(index)
    k = cfg["k"]
    t0 = time.time()
    ref = H.oracle_verify(oi["z_t"], oi["z_d"], oi["x"], seed=0, step=0)
    got = H.gpu_verify(d["z_t"], d["z_d"], d["x"], seed=0, step=0)
    n_tie, n_edge = H.assert_verify(got, ref, k)
    print(f"  verify (gamma = k) ok: near-tie {n_tie}, near-cdf-edge {n_edge}, "
          f"mean accepted {ref['n_accept'].mean():.2f} ({time.time() - t0:.1f}s)", flush=True)
    rg, _, _ = O.select_length(rp, lat)
    ref = H.oracle_verify(oi["z_t"], oi["z_d"], oi["x"], gamma=rg, seed=1, step=3)
    got = H.gpu_verify(d["z_t"], d["z_d"], d["x"], gamma=rg, seed=1, step=3)
    n_tie, n_edge = H.assert_verify(got, ref, k)
    print(f"  verify (selected gamma, mean {rg.mean():.2f}) ok: near-tie {n_tie}, near-cdf-edge {n_edge}",
          flush=True)
    H.assert_verify(H.gpu_verify_chained(d["z_t"], d["z_d"], d["z_c"], d["x"], gamma=rg, seed=1, step=3), ref, k)


def test_full_config5_ragged_chain():
    cfg, d, oi, rp, lat = _stage_isolated(4)
    B, k = cfg["B"], cfg["k"]
    rg, ro, rm = O.select_length(rp, lat)
    assert 0 < rm < B * k, "the latency table should make the selection non-trivial"
    # the caller packs the target rows of the selected positions + bonus row
    packed = torch.cat([d["z_t"][b, :rg[b] + 1] for b in range(B)]).contiguous()
    packed_np = np.concatenate([oi["z_t"][b, :rg[b] + 1] for b in range(B)])
    assert packed.shape[0] == ro[-1]
    ref = H.oracle_verify(packed_np, oi["z_d"], oi["x"], gamma=rg, t_offsets=ro, seed=5, step=2)
    got = H.gpu_verify(packed, d["z_d"], d["x"], gamma=rg, t_offsets=ro, seed=5, step=2)
    n_tie, n_edge = H.assert_verify(got, ref, k)
    full = int((ref["n_accept"] == rg).sum())
    early = int(((ref["n_accept"] < rg) & (rg > 0)).sum())
    print(f"  ragged verify ok: sum gamma {rm}, packed rows {ro[-1]}, full-accept rows {full}, "
          f"early-stop rows {early}, gamma=0 rows {int((rg == 0).sum())}, near-tie {n_tie}, "
          f"near-cdf-edge {n_edge}", flush=True)
    # dense layout with the same lengths must agree with the packed one
    got_dense = H.gpu_verify(d["z_t"], d["z_d"], d["x"], gamma=rg, seed=5, step=2)
    assert np.array_equal(got_dense["tokens"], got["tokens"])
    assert np.array_equal(got_dense["n_accept"], got["n_accept"])
    # the chained call (draft normalisers from sv_row_stats, only the packed target rows swept)
    got_chained = H.gpu_verify_chained(packed, d["z_d"], d["z_c"], d["x"], gamma=rg, t_offsets=ro, seed=5, step=2)
    H.assert_verify(got_chained, ref, k)


def test_full_config_warped_compacted_ragged():
    """Config 5 at full size with sampling warps on compacted supports: lengths from
    sv_select_length, target supports compacted from the packed target rows.  Every
    sequence is compared with the dense warped entry points and with the oracle
    itself (the oracle warps and verifies the rows each sequence needs)."""
    from oracle import warp_oracle as W
    P = H.sv()
    cfg = svgen.make_config(4, device="cuda")
    B, k, V = cfg["B"], cfg["k"], cfg["V"]
    T, K, Pp, cap = float(np.float32(0.7)), 20, 0.8, 64
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    sup_d, sup_c = P.Supports(B * k, cap), P.Supports(B * k, cap)
    cut_d, cut_c = f32(B * k), f32(B * k)
    wf_d, wf_c = i32(B * k), i32(B * k)
    P.sv_warp_compact(cfg["z_d"], T, K, Pp, sup_d, cut_d, wf_d)
    P.sv_warp_compact(cfg["z_c"], T, K, Pp, sup_c, cut_c, wf_c)
    lse_d, lse_c, S, A, p_hat = (f32(B, k) for _ in range(5))
    P.sv_row_stats_sparse(sup_d, sup_c, cfg["x"], V, lse_d, lse_c, S, A)
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = H.dev(svgen.latency_table(B * k), torch.float32)
    gamma, offs, total = i32(B), i32(B + 1), i32(1)
    P.sv_accept_estimate(S, A, H.dev(edges_s), H.dev(edges_a), H.dev(table), p_hat, None)
    P.sv_select_length(p_hat, lat, P.SV_BATCH_GREEDY, gamma, offs, total)
    torch.cuda.synchronize()
    g = gamma.cpu().numpy()
    o = offs.cpu().numpy()
    assert (sup_d.count.cpu().numpy() > 0).all() and int(total.item()) == int(g.sum())
    # pack the target rows of the selected positions plus the bonus row
    z_tp = torch.cat([cfg["z_t"][b, :g[b] + 1] for b in range(B)], dim=0).contiguous()
    rows_t = z_tp.shape[0]
    assert rows_t == o[-1]
    sup_t, cut_t, wf_t = P.Supports(rows_t, cap), f32(rows_t), i32(rows_t)
    P.sv_warp_compact(z_tp, T, K, Pp, sup_t, cut_t, wf_t)
    res = {}
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    for mode in ("sparse", "dense"):
        tokens, n_acc, flags, ratio = i32(B, k + 1), i32(B), i32(B), f32(B, k)
        if mode == "sparse":
            P.sv_verify_sample_sparse(sup_t, offs, sup_d, cfg["x"], gamma, V, 9, 2, tokens, n_acc, flags, ratio)
        else:
            P.sv_verify_sample_warped(z_tp, offs, cfg["z_d"], cfg["x"], gamma, T, cut_t, T, cut_d, 9, 2, tokens, n_acc,
                                      flags, ratio, ws)
        torch.cuda.synchronize()
        res[mode] = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
                         flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
    s, d = res["sparse"], res["dense"]
    assert not (s["flags"] & 32).any()
    near = ((s["flags"] | d["flags"]) & (O.FLAG_NEAR_TIE | O.FLAG_NEAR_CDF_EDGE)) != 0
    ok = ~near
    assert np.array_equal(s["n_accept"][ok], d["n_accept"][ok]) and np.array_equal(s["tokens"][ok], d["tokens"][ok])
    assert near.sum() <= 6
    # the oracle on every sequence (the rows it needs only)
    zt_bits, zd_bits = svgen.to_numpy_bits(z_tp), svgen.to_numpy_bits(cfg["z_d"])
    x = cfg["x"].cpu().numpy()
    wt, wd = wf_t.cpu().numpy().astype(np.uint32), wf_d.cpu().numpy().astype(np.uint32).reshape(B, k)
    checked = 0
    for b in range(B):
        rows = slice(o[b], o[b + 1])
        nd = int(g[b])
        y_t, _, f_t = W.warp_rows(zt_bits[rows], T, K, Pp)
        y_d = np.full((1, k, V), -np.inf)                 # draft rows beyond the verified length are never read
        f_d = np.zeros(k, dtype=np.uint32)
        if nd:
            yd, _, fd = W.warp_rows(zd_bits[b, :nd], T, K, Pp)
            y_d[0, :nd], f_d[:nd] = yd, fd
        if ((f_t | wt[rows]) & O.FLAG_NEAR_TIE).any() or ((f_d | wd[b]) & O.FLAG_NEAR_TIE)[:nd].any():
            continue
        # the oracle addresses its uniforms by the sequence index: hand it those of sequence b
        from oracle import philox as OP
        ua, _ = OP.sv_uniforms(9, 2, np.full((1, k), b), np.arange(k)[None, :])
        _, us_full = OP.sv_uniforms(9, 2, np.full((1, k + 1), b), np.arange(k + 1)[None, :])
        ref = H.oracle_verify(y_t, y_d, x[b:b + 1], gamma=g[b:b + 1], t_offsets=np.array([0, g[b] + 1], np.int32),
                              uniforms=(ua, us_full))
        got = {n: v[b:b + 1] for n, v in s.items()}
        H.assert_verify(got, ref, k)
        checked += 1
    assert checked >= B - 6
    print(f"\n  cfg5 warped, compacted: mean gamma {g.mean():.2f}, near flags {int(near.sum())}, "
          f"oracle-checked sequences {checked}", flush=True)


def test_large_batch_chain():
    """B = 512, k = 16 (8192 keys: the largest batch sv_select_length takes) through
    the whole chain.  The estimate and the lengths are checked on the whole batch
    (oracle rule on the GPU's own float32 S, A), the indicators and the verification
    on a sample of sequences."""
    from oracle import philox as OP
    P = H.sv()
    B, k, V = 512, 16, 32000
    cfg = svgen.make_config(1, seed=31337, B=B, k=k, V=V, dtype="bf16", device="cuda")
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    lse_d, lse_c, S, A, p_hat, ratio = (f32(B, k) for _ in range(6))
    gamma, offs, total = i32(B), i32(B + 1), i32(1)
    tokens, n_acc, flags = i32(B, k + 1), i32(B), i32(B)
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = svgen.latency_table(B * k)
    P.sv_row_stats(cfg["z_d"], cfg["z_c"], cfg["x"], lse_d, lse_c, S, A, None, None, ws)
    P.sv_accept_estimate(S, A, H.dev(edges_s), H.dev(edges_a), H.dev(table), p_hat, None)
    P.sv_select_length(p_hat, H.dev(lat, torch.float32), P.SV_BATCH_GREEDY, gamma, offs, total)
    P.sv_verify_sample(cfg["z_t"], None, cfg["z_d"], cfg["x"], gamma, 5, 6, tokens, n_acc, flags, ratio, ws)
    torch.cuda.synchronize()
    p_ref, _ = O.accept_estimate(S.cpu().numpy(), A.cpu().numpy(), edges_s, edges_a, table)
    assert np.array_equal(p_hat.cpu().numpy(), p_ref)
    rg, ro, rm = O.select_length(p_ref, lat, O.MODE_BATCH_GREEDY)
    assert int(total.item()) == rm and np.array_equal(gamma.cpu().numpy(), rg) and np.array_equal(offs.cpu().numpy(), ro)
    got_all = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
                   flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
    x = cfg["x"].cpu().numpy()
    for b in (0, 1, 255, 256, 511):
        zt = svgen.to_numpy_bits(cfg["z_t"][b:b + 1])
        zd = svgen.to_numpy_bits(cfg["z_d"][b:b + 1])
        zc = svgen.to_numpy_bits(cfg["z_c"][b:b + 1])
        r = O.row_stats(zd, zc, x[b:b + 1])
        assert H.close(S.cpu().numpy()[b], r["S"][0], H.REL).all() and H.close(A.cpu().numpy()[b], r["A"][0], H.REL, 1e-30).all()
        ua, _ = OP.sv_uniforms(5, 6, np.full((1, k), b), np.arange(k)[None, :])
        _, us = OP.sv_uniforms(5, 6, np.full((1, k + 1), b), np.arange(k + 1)[None, :])
        ref = H.oracle_verify(zt, zd, x[b:b + 1], gamma=rg[b:b + 1], uniforms=(ua, us))
        H.assert_verify({n: v[b:b + 1] for n, v in got_all.items()}, ref, k)
