"""GPU parity for the profile-construction / information-gain pass."""
import numpy as np
import pytest
import torch

import svgen
from oracle import profile_oracle as PO
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu


def _gpu_accept_ratio(z_t, z_d, x):
    P = H.sv()
    B, k, V = z_d.shape
    ratio = torch.full((B, k), -3.0, dtype=torch.float32, device="cuda")
    flags = torch.full((B, k), 77, dtype=torch.int32, device="cuda")
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(z_d))
    P.sv_accept_ratio(z_t, z_d, x, ratio, flags, ws)
    torch.cuda.synchronize()
    return ratio.cpu().numpy(), flags.cpu().numpy().astype(np.uint32)


@pytest.mark.parametrize("idx,B,k,V,dtype", [(1, 4, 5, 32000, "bf16"), (0, 2, 3, 4099, "f32"),
                                             (2, 3, 4, 20000, "bf16"), (3, 2, 8, 16392, "bf16")])
def test_accept_ratio_every_position(idx, B, k, V, dtype):
    cfg = svgen.make_config(idx, B=B, k=k, V=V, dtype=dtype)
    cfg["x"][0, 1] = V + 5                                  # impossible token
    cfg["z_d"][B - 1, 0, 3] = float("nan")                  # bad draft row
    oi = H.oracle_inputs(cfg)
    ref, rflags = PO.accept_probability_ratio(oi["z_t"], oi["z_d"], oi["x"])
    for z_t in (cfg["z_t"], cfg["z_t"][:, :k].contiguous()):   # with and without the bonus row
        got, gflags = _gpu_accept_ratio(z_t.cuda(), cfg["z_d"].cuda(), cfg["x"].cuda())
        assert np.array_equal(gflags, rflags)
        assert H.close(got, ref, H.REL, 1e-30).all(), (got, ref)


def test_quantile_edges_exact():
    P = H.sv()
    rng = np.random.default_rng(0)
    for n, n_bins in ((1, 4), (7, 3), (512, 16), (4096, 17), (8192, 20), (5000, 1), (0, 5)):
        v = (rng.random(n) ** 2).astype(np.float32)
        if n > 10:
            v[::37] = np.nan
            v[5:5 + n // 3] = 1.0                           # heavy ties, like the saturated A
        ref = PO.quantile_edges(v, n_bins)
        edges = torch.full((n_bins + 1,), -9.0, dtype=torch.float32, device="cuda")
        vals = torch.from_numpy(v).cuda() if n else torch.empty(0, dtype=torch.float32, device="cuda")
        P.sv_quantile_edges(vals, n_bins, 0.0, 1.0, edges)
        torch.cuda.synchronize()
        assert np.array_equal(edges.cpu().numpy(), ref), (n, n_bins)


def _gpu_profile(S, A, ratio, edges_s, edges_a, n_x, batches=1):
    P = H.sv()
    n_s, n_a = len(edges_s) - 1, len(edges_a) - 1
    counts = torch.zeros((n_s, n_a, n_x), dtype=torch.int32, device="cuda")
    sum_x = torch.zeros((n_s, n_a), dtype=torch.float64, device="cuda")
    es, ea = H.dev(edges_s), H.dev(edges_a)
    for part in np.array_split(np.arange(S.size), batches):
        if part.size:
            P.sv_profile_accumulate(H.dev(S[part]), H.dev(A[part]), H.dev(ratio[part]), es, ea, n_x, counts, sum_x)
    table = torch.full((n_s, n_a), -1.0, dtype=torch.float32, device="cuda")
    info = torch.full((3,), -1.0, dtype=torch.float64, device="cuda")
    P.sv_profile_finalize(counts, sum_x, table, info)
    torch.cuda.synchronize()
    return counts.cpu().numpy(), sum_x.cpu().numpy(), table.cpu().numpy(), info.cpu().numpy()


def test_accumulate_and_finalize():
    rng = np.random.default_rng(1)
    for n, n_s, n_a, n_x in ((5000, 5, 5, 10), (300, 16, 17, 8), (20, 20, 20, 4), (0, 3, 3, 5)):
        S = rng.random(n).astype(np.float32)
        A = np.minimum(1, 1.5 * rng.random(n)).astype(np.float32)
        ratio = (1.7 * rng.random(n)).astype(np.float32)
        if n > 10:
            S[3], A[4], ratio[5] = np.nan, np.nan, np.nan
            ratio[6], ratio[7] = 1.0, 0.0
        edges_s = np.sort(np.concatenate([[0, 1], rng.random(n_s - 1)])).astype(np.float32)
        edges_a = np.linspace(0, 1, n_a + 1).astype(np.float32)
        rc, rs = PO.accumulate(S, A, ratio, edges_s, edges_a, n_x)
        rt, rinfo = PO.finalize(rc, rs)
        for batches in (1, 3):
            gc, gs, gt, ginfo = _gpu_profile(S, A, ratio, edges_s, edges_a, n_x, batches)
            assert np.array_equal(gc.astype(np.int64), rc)
            assert np.allclose(gs, rs, rtol=1e-12, atol=1e-300)
            assert np.allclose(gt, rt, rtol=2e-7, atol=0)       # fp32 rounding of an fp64 mean
            assert np.allclose(ginfo, np.array(rinfo), rtol=1e-11, atol=1e-12)


def test_profile_pass_end_to_end_and_lookup():
    """row_stats -> accept_ratio -> adaptive edges -> histogram -> table + information gain,
    all on the GPU, against the oracle chain; then the table feeds sv_accept_estimate."""
    P = H.sv()
    cfg = svgen.make_config(1, B=16, k=8, V=8192, dtype="bf16", seed=4242)
    d = {n: cfg[n].cuda() for n in ("z_t", "z_d", "z_c", "x")}
    oi = H.oracle_inputs(cfg)
    B, k, V = 16, 8, 8192
    stats = H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl=False)
    ratio, _ = _gpu_accept_ratio(d["z_t"], d["z_d"], d["x"])
    r = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
    rr, _ = PO.accept_probability_ratio(oi["z_t"], oi["z_d"], oi["x"])
    S32, A32, X32 = r["S"].astype(np.float32), r["A"].astype(np.float32), rr.astype(np.float32)
    assert H.close(stats["S"], S32).all() and H.close(ratio, X32, H.REL, 1e-30).all()
    # from here on both sides start from the oracle's S, A, X (stage isolation)
    n_s, n_a, n_x = 6, 5, 10
    es_ref, ea_ref = PO.quantile_edges(S32, n_s), PO.quantile_edges(A32, n_a)
    es = torch.empty(n_s + 1, dtype=torch.float32, device="cuda")
    ea = torch.empty(n_a + 1, dtype=torch.float32, device="cuda")
    P.sv_quantile_edges(H.dev(S32.ravel()), n_s, 0.0, 1.0, es)
    P.sv_quantile_edges(H.dev(A32.ravel()), n_a, 0.0, 1.0, ea)
    torch.cuda.synchronize()
    assert np.array_equal(es.cpu().numpy(), es_ref) and np.array_equal(ea.cpu().numpy(), ea_ref)
    rc, rs = PO.accumulate(S32, A32, X32, es_ref, ea_ref, n_x)
    rt, rinfo = PO.finalize(rc, rs)
    gc, gs, gt, ginfo = _gpu_profile(S32.ravel(), A32.ravel(), X32.ravel(), es_ref, ea_ref, n_x)
    assert np.array_equal(gc.astype(np.int64), rc) and np.allclose(gt, rt, rtol=2e-7)
    assert np.allclose(ginfo, np.array(rinfo), rtol=1e-11, atol=1e-12)
    assert ginfo[2] > 0.0                       # observing (S, A) tells something about X
    print(f"\n  synthetic profile: H(X)={ginfo[0]:.3f} H(X|S,A)={ginfo[1]:.3f} I={ginfo[2]:.3f} bits")
    p_ref, _ = O.accept_estimate(S32, A32, es_ref, ea_ref, rt)
    p_got, _ = H.gpu_accept_estimate(S32, A32, es_ref, ea_ref, gt)
    same_table = np.array_equal(gt, rt)
    assert (not same_table) or np.array_equal(p_got, p_ref)
