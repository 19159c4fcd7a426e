"""sv_estimate_select (the estimate lookup and the length selection in one launch) against
the oracle's two functions and against the two separate calls: estimates, edge flags,
lengths, offsets and totals are integers or table entries, so everything is compared
bit for bit."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu


def _fused(S, A, edges_s, edges_a, table, lat, mode, with_flag=True):
    P = H.sv()
    S_d, A_d = H.dev(S, torch.float32), H.dev(A, torch.float32)
    B, k = S_d.shape
    p_hat = torch.full((B, k), -3.0, dtype=torch.float32, device="cuda")
    flag = torch.full((B, k), 9, dtype=torch.uint8, device="cuda") if with_flag else None
    gamma = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    offs = torch.full((B + 1,), -9, dtype=torch.int32, device="cuda")
    total = torch.full((1,), -9, dtype=torch.int32, device="cuda")
    P.sv_estimate_select(S_d, A_d, H.dev(edges_s), H.dev(edges_a), H.dev(table), H.dev(lat, torch.float32), mode,
                         p_hat, gamma, offs, total, edge_flag=flag)
    torch.cuda.synchronize()
    return (p_hat.cpu().numpy(), None if flag is None else flag.cpu().numpy(), gamma.cpu().numpy(),
            offs.cpu().numpy(), int(total.item()))


@pytest.mark.parametrize("B,k,n_s,n_a", [(1, 4, 10, 10), (8, 8, 5, 5), (64, 8, 10, 10), (64, 16, 20, 20),
                                         (3, 1, 1, 1), (37, 5, 16, 17), (512, 16, 10, 10), (7, 64, 272, 1)])
def test_estimate_select_matches_the_oracle_and_the_two_calls(B, k, n_s, n_a):
    rng = np.random.default_rng(1000 * B + k)
    edges_s = np.sort(np.concatenate([[0.0, 1.0], rng.random(n_s - 1)])).astype(np.float32)
    edges_a = np.sort(np.concatenate([[0.0, 1.0], rng.random(n_a - 1)])).astype(np.float32)
    table = rng.random((n_s, n_a)).astype(np.float32)
    for trial in range(3):
        S = rng.random((B, k)).astype(np.float32)
        A = np.minimum(1.0, rng.random((B, k)) * 1.3).astype(np.float32)
        if trial == 1:                                   # values on and next to the edges, out of range, NaN
            pick = rng.random((B, k)) < 0.3
            S[pick] = rng.choice(edges_s, size=int(pick.sum()))
            A[rng.random((B, k)) < 0.1] = np.nextafter(np.float32(edges_a[min(1, n_a)]), np.float32(0))
            S[rng.random((B, k)) < 0.05] = np.nan
            A[rng.random((B, k)) < 0.05] = 1.5
            S[rng.random((B, k)) < 0.05] = -0.25
        if trial == 2:
            table = np.round(table * 4) / 4              # ties between the products
            table = table.astype(np.float32)
        lat_b = svgen.latency_table(B * k, t0=float(rng.uniform(0.1, 30)), d=0.08, m0=max(1, B * k // 4))
        rp, rflag = O.accept_estimate(S, A, edges_s, edges_a, table)
        for mode, lat in ((O.MODE_BATCH_GREEDY, lat_b), (O.MODE_PER_SEQUENCE, lat_b[:k + 1])):
            rg, ro, rm = O.select_length(rp, lat, mode)
            p, f, g, o, m = _fused(S, A, edges_s, edges_a, table, lat, mode)
            assert np.array_equal(p, rp, equal_nan=True)
            assert np.array_equal(f.astype(bool), np.asarray(rflag).astype(bool))
            assert m == rm and np.array_equal(g, rg) and np.array_equal(o, ro)
            # the two separate calls give the same
            p2, f2 = H.gpu_accept_estimate(S, A, edges_s, edges_a, table)
            g2, o2, m2 = H.gpu_select_length(p2, lat, mode)
            assert np.array_equal(p, p2, equal_nan=True) and np.array_equal(f, f2)
            assert m == m2 and np.array_equal(g, g2) and np.array_equal(o, o2)
    p, f, g, o, m = _fused(S, A, edges_s, edges_a, table, lat_b, O.MODE_BATCH_GREEDY, with_flag=False)
    assert f is None and np.array_equal(p, rp, equal_nan=True)


def test_estimate_select_in_the_chained_step():
    """Three calls instead of four on device buffers (config 2 shape): row statistics,
    estimate + selection, chained verification of the selected lengths."""
    P = H.sv()
    B, k, V = 8, 8, 32000
    cfg = svgen.make_config(1, seed=77, B=B, k=k, V=V, dtype="bf16", device="cuda")
    oi = H.oracle_inputs(cfg)
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = svgen.latency_table(B * k)
    f = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    i = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    lse_d, lse_c, S, A, p_hat, ratio = (f(B, k) for _ in range(6))
    gamma, offs, total, tokens, n_acc, flags = i(B), i(B + 1), i(1), i(B, k + 1), i(B), i(B)
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    P.sv_row_stats(cfg["z_d"], cfg["z_c"], cfg["x"], lse_d, lse_c, S, A, None, None, ws)
    P.sv_estimate_select(S, A, H.dev(edges_s), H.dev(edges_a), H.dev(table), H.dev(lat), P.SV_BATCH_GREEDY, p_hat,
                         gamma, offs, total)
    P.sv_verify_sample_chained(cfg["z_t"], None, cfg["z_d"], cfg["x"], gamma, 4, 2, tokens, n_acc, flags, ratio, ws)
    torch.cuda.synchronize()
    r = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
    rp, _ = O.accept_estimate(r["S"].astype(np.float32), r["A"].astype(np.float32), edges_s, edges_a, table)
    rg, ro, rm = O.select_length(rp, lat)
    assert np.array_equal(p_hat.cpu().numpy(), rp) and np.array_equal(gamma.cpu().numpy(), rg)
    assert np.array_equal(offs.cpu().numpy(), ro) and int(total.item()) == rm
    ref = H.oracle_verify(oi["z_t"], oi["z_d"], oi["x"], gamma=rg, seed=4, step=2)
    got = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
               flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
    H.assert_verify(got, ref, k)
