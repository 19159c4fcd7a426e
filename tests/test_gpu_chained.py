"""sv_verify_sample_chained (draft normalisers taken from what sv_row_stats left in
the workspace; only the target rows are swept) against the oracle, by the same
parity rule as sv_verify_sample, and against sv_verify_sample itself.  Also the
checks of the hand-over: a workspace that holds no statistics pass, or one of
other arguments, must be recognised (SV_FLAG_NO_CHAIN), never used."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O
from oracle import warp_oracle as W

import harness as H

pytestmark = pytest.mark.gpu

NO_CHAIN = 64


def _stats_outputs(B, k):
    mk = lambda: torch.full((B, k), -7.0, dtype=torch.float32, device="cuda")
    return dict(lse_d=mk(), lse_c=mk(), S=mk(), A=mk())


def _verify_outputs(B, k):
    return dict(tokens=torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda"),
                n_accept=torch.full((B,), -5, dtype=torch.int32, device="cuda"),
                flags=torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda"),
                ratio=torch.full((B, k), -5.0, dtype=torch.float32, device="cuda"))


def _host(out):
    r = {n: t.cpu().numpy() for n, t in out.items()}
    r["flags"] = r["flags"].astype(np.uint32)
    return r


def _chained(cfg, gamma=None, t_offsets=None, z_t=None, seed=0, step=0, ws=None, stats=True, z_d_verify=None,
             x_verify=None):
    """sv_row_stats, then sv_verify_sample_chained on the same workspace."""
    P = H.sv()
    z_d, z_c, x = cfg["z_d"], cfg["z_c"], cfg["x"]
    z_t = cfg["z_t"] if z_t is None else z_t
    B, k, V = z_d.shape
    if ws is None:
        ws = torch.zeros(P.sv_workspace_bytes(B, k, V, P.binding._dtype_tag(z_d)), dtype=torch.uint8, device="cuda")
    st = _stats_outputs(B, k)
    if stats:
        P.sv_row_stats(z_d, z_c, x, st["lse_d"], st["lse_c"], st["S"], st["A"], None, None, ws)
    out = _verify_outputs(B, k)
    g = None if gamma is None else H.dev(gamma, torch.int32)
    o = None if t_offsets is None else H.dev(t_offsets, torch.int32)
    P.sv_verify_sample_chained(z_t, o, z_d if z_d_verify is None else z_d_verify, x if x_verify is None else x_verify,
                               g, seed, step, out["tokens"], out["n_accept"], out["flags"], out["ratio"], ws)
    torch.cuda.synchronize()
    return _host(out)


def _same_as_unchained(got, plain):
    """Both paths run the same kernels on normalisers that may differ in their last bits:
    identical integers wherever neither raised a near-tie / near-edge flag."""
    soft = O.FLAG_NEAR_TIE | O.FLAG_NEAR_CDF_EDGE
    clear = ((got["flags"] | plain["flags"]) & soft) == 0
    assert np.array_equal(got["n_accept"][clear], plain["n_accept"][clear])
    assert np.array_equal(got["tokens"][clear], plain["tokens"][clear])
    assert np.array_equal(got["flags"][clear], plain["flags"][clear])
    ev = ~np.isnan(plain["ratio"][clear])
    assert np.array_equal(np.isnan(got["ratio"][clear]), ~ev)
    assert H.close(got["ratio"][clear][ev], plain["ratio"][clear][ev], 1e-6, 1e-30).all()
    return int(clear.sum())


# (config index, B, k, V, dtype): aligned bf16, the headline vocabulary, fp32, rows that are not
# whole 16-byte vectors (the plain two-sweep statistics kernel), a vocabulary below one chunk
CASES = [(1, 6, 5, 32000, "bf16"), (3, 3, 4, 152064, "bf16"), (0, 3, 3, 40000, "f32"), (2, 4, 3, 20011, "bf16"),
         (0, 2, 2, 4099, "f32"), (1, 2, 1, 777, "bf16")]


@pytest.mark.parametrize("idx,B,k,V,dtype", CASES)
def test_chained_matches_oracle_and_unchained(idx, B, k, V, dtype):
    cfg = svgen.make_config(idx, seed=500 + idx, B=B, k=k, V=V, dtype=dtype, device="cuda")
    inp = H.oracle_inputs(cfg)
    ties = clear = 0
    for step in range(4):
        got = _chained(cfg, seed=31, step=step)
        assert (got["flags"] & NO_CHAIN == 0).all()
        ref = H.oracle_verify(inp["z_t"], inp["z_d"], inp["x"], seed=31, step=step)
        t, _ = H.assert_verify(got, ref, k)
        ties += t
        plain = H.gpu_verify(cfg["z_t"], cfg["z_d"], cfg["x"], seed=31, step=step)
        clear += _same_as_unchained(got, plain)
    assert ties <= 1 and clear >= 3 * B


def test_chained_ragged_lengths_dense_and_packed():
    B, k, V = 7, 6, 50000
    cfg = svgen.make_config(3, seed=611, B=B, k=k, V=V, dtype="bf16", device="cuda")
    inp = H.oracle_inputs(cfg)
    gamma = np.array([0, 6, 3, 1, 6, 0, 4], dtype=np.int32)
    offs = np.concatenate([[0], np.cumsum(gamma + 1)]).astype(np.int32)
    rows = [cfg["z_t"][b, i] for b in range(B) for i in range(gamma[b] + 1)]
    packed = torch.stack(rows).contiguous()
    for step in range(3):
        ref = H.oracle_verify(inp["z_t"], inp["z_d"], inp["x"], gamma=gamma, seed=8, step=step)
        dense = _chained(cfg, gamma=gamma, seed=8, step=step)
        H.assert_verify(dense, ref, k)
        pk = _chained(cfg, gamma=gamma, t_offsets=offs, z_t=packed, seed=8, step=step)
        H.assert_verify(pk, ref, k)
        for name in ("tokens", "n_accept", "flags"):
            assert np.array_equal(dense[name], pk[name]), name


def test_chained_bad_rows_and_tokens_as_unchained():
    """NaN / +inf / all -inf draft rows, a bad companion row (must not touch verification) and
    drafted tokens out of range: the chained call flags exactly what the plain call flags."""
    B, k, V = 6, 3, 9000
    cfg = svgen.make_config(1, seed=712, B=B, k=k, V=V, dtype="bf16", device="cuda")
    z_d, z_c, x = cfg["z_d"].clone(), cfg["z_c"].clone(), cfg["x"].clone()
    z_d[0, 1, 17] = float("nan")
    z_d[1, 0, 5] = float("inf")
    z_d[2, 2, :] = float("-inf")
    z_c[3, 0, 3] = float("nan")
    x[4, 1] = V
    x[5, 0] = -1
    bad = dict(cfg, z_d=z_d, z_c=z_c, x=x)
    got = _chained(bad, seed=3, step=1)
    plain = H.gpu_verify(cfg["z_t"], z_d, x, seed=3, step=1)
    assert (got["flags"] & NO_CHAIN == 0).all()
    for name in ("tokens", "n_accept", "flags"):
        assert np.array_equal(got[name], plain[name]), (name, got[name], plain[name])
    ref = H.oracle_verify(svgen.to_numpy_bits(cfg["z_t"]), svgen.to_numpy_bits(z_d), x.cpu().numpy(), seed=3, step=1)
    H.assert_verify(got, ref, k)


def _assert_no_chain(got, B):
    assert ((got["flags"] & NO_CHAIN) != 0).all(), got["flags"]
    assert (got["n_accept"] == 0).all()
    assert (got["tokens"][:, 0] >= 0).all() and (got["tokens"][:, 1:] == -1).all()


def test_workspace_without_or_with_another_statistics_pass_is_recognised():
    B, k, V = 4, 3, 12000
    P = H.sv()
    cfg = svgen.make_config(1, seed=813, B=B, k=k, V=V, dtype="bf16", device="cuda")
    nbytes = P.sv_workspace_bytes(B, k, V, P.SV_BF16)
    # no statistics pass at all: zeros, then arbitrary bytes
    _assert_no_chain(_chained(cfg, stats=False), B)
    junk = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda")
    _assert_no_chain(_chained(cfg, stats=False, ws=junk), B)
    # a pass on another draft tensor / other tokens (same values elsewhere in memory: the names differ)
    _assert_no_chain(_chained(cfg, z_d_verify=cfg["z_d"].clone()), B)
    _assert_no_chain(_chained(cfg, x_verify=cfg["x"].clone()), B)
    # a pass of another shape on the same workspace
    ws = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    small = svgen.make_config(1, seed=814, B=B, k=k - 1, V=V, dtype="bf16", device="cuda")
    st = _stats_outputs(B, k - 1)
    P.sv_row_stats(small["z_d"], small["z_c"], small["x"], st["lse_d"], st["lse_c"], st["S"], st["A"], None, None, ws)
    _assert_no_chain(_chained(cfg, stats=False, ws=ws), B)
    # and the right pass afterwards is taken again; gamma = 0 needs no draft row but still reports the state
    good = _chained(cfg, ws=ws)
    assert (good["flags"] & NO_CHAIN == 0).all()
    zero = _chained(cfg, stats=False, gamma=np.zeros(B, dtype=np.int32))
    assert ((zero["flags"] & NO_CHAIN) != 0).all() and (zero["tokens"][:, 0] >= 0).all()


def test_chained_warped_matches_oracle_and_checks_the_draft_warp():
    P = H.sv()
    B, k, V = 4, 3, 32000
    cfg = svgen.make_config(1, seed=915, B=B, k=k, V=V, dtype="bf16", device="cuda")
    inp = H.oracle_inputs(cfg)
    f32 = lambda T: float(np.float32(T))
    Tt, Td, Tc = f32(0.7), f32(0.95), f32(0.6)
    y_t, cut_t, _ = W.warp_rows(inp["z_t"], Tt, 20, 0.8)
    y_d, cut_d, _ = W.warp_rows(inp["z_d"], Td, 20, 0.6)
    _, cut_c, _ = W.warp_rows(inp["z_c"], Tc, 0, 0.9)
    c_t, c_d, c_c = (H.dev(np.asarray(c, dtype=np.float32)) for c in (cut_t, cut_d, cut_c))
    ws = torch.zeros(P.sv_workspace_bytes(B, k, V, P.SV_BF16), dtype=torch.uint8, device="cuda")
    st = _stats_outputs(B, k)
    P.sv_row_stats_warped(cfg["z_d"], cfg["z_c"], cfg["x"], Td, c_d, Tc, c_c, st["lse_d"], st["lse_c"], st["S"],
                          st["A"], None, None, ws)

    def run(step, Td_=Td, c_d_=c_d):
        out = _verify_outputs(B, k)
        P.sv_verify_sample_warped_chained(cfg["z_t"], None, cfg["z_d"], cfg["x"], None, Tt, c_t, Td_, c_d_, 5, step,
                                          out["tokens"], out["n_accept"], out["flags"], out["ratio"], ws)
        torch.cuda.synchronize()
        return _host(out)

    for step in range(3):
        got = run(step)
        assert (got["flags"] & NO_CHAIN == 0).all()
        H.assert_verify(got, H.oracle_verify(y_t, y_d, inp["x"], seed=5, step=step), k)
    # another draft temperature, or another cutoff array, is not what the statistics pass used
    _assert_no_chain(run(0, Td_=f32(0.9)), B)
    _assert_no_chain(run(0, c_d_=c_d.clone()), B)
    # nor is the unwarped call
    out = _verify_outputs(B, k)
    P.sv_verify_sample_chained(cfg["z_t"], None, cfg["z_d"], cfg["x"], None, 5, 0, out["tokens"], out["n_accept"],
                               out["flags"], out["ratio"], ws)
    torch.cuda.synchronize()
    _assert_no_chain(_host(out), B)


def test_chained_full_size_headline_configuration():
    """Config 4 at full size, in the launch configuration the benchmark times: every sequence
    against the plain call, a sample of sequences against the oracle."""
    cfg = svgen.make_config(3, seed=1003, device="cuda")
    B, k, V = cfg["z_d"].shape
    got = _chained(cfg, seed=0, step=0)
    plain = H.gpu_verify(cfg["z_t"], cfg["z_d"], cfg["x"], seed=0, step=0)
    assert (got["flags"] & NO_CHAIN == 0).all()
    assert _same_as_unchained(got, plain) >= B - 4
    pick = [0, 7, 31, 63]
    inp = H.oracle_inputs(cfg)
    ref = H.oracle_verify(inp["z_t"][pick], inp["z_d"][pick], inp["x"][pick], seed=0, step=0,
                          uniforms=H.uniforms_of(pick, k))
    sub = {n: got[n][pick] for n in got}
    H.assert_verify(sub, ref, k)
