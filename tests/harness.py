"""Helpers for the GPU parity tests: run the HIP path through the C ABI on
torch tensors, run the oracle on the same stored values, and compare by the
parity rule (integers bit-exact off the flagged near-tie bands, floats within
1e-5 relative)."""
from __future__ import annotations

import numpy as np
import torch

import svgen
from oracle import sv_oracle as O

REL = 1e-5
# Absolute resolution of the dense HIP path's cumulative sampling weights (fp32 probabilities,
# each within 2.5e-7 relative: at most 5e-7 on a cumulative sum and on the threshold).  The
# oracle, in fp64, has no such limit; it is handed this band so that its FLAG_NEAR_CDF_EDGE and
# its admissible sets cover what the HIP path cannot resolve.  Compacted supports hold fp64
# probabilities and would do with 0; the same band is used for all paths for simplicity.
GPU_CDF_ABS_BAND = 1e-6


def oracle_verify(*args, **kw):
    """The oracle's verification step with the comparison band of the HIP path."""
    kw.setdefault("cdf_abs_band", GPU_CDF_ABS_BAND)
    return O.verify_sample(*args, **kw)


def sv():
    import paper_2509_24328_amd as P
    return P


def dev(a, dtype=None):
    t = torch.as_tensor(a)
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda().contiguous()


# ------------------------------------------------------------------ GPU runs
def gpu_row_stats(z_d, z_c, x, with_kl=True):
    P = sv()
    B, k, V = z_d.shape
    mk = lambda: torch.full((B, k), -7.0, dtype=torch.float32, device="cuda")
    out = dict(lse_d=mk(), lse_c=mk(), S=mk(), A=mk(), KL=mk() if with_kl else None,
               H_d=mk() if with_kl else None, pd_x=mk(),
               flags=torch.full((B, k), 0xFFFF, dtype=torch.int32, device="cuda"))
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(z_d))
    P.sv_row_stats(z_d, z_c, x, out["lse_d"], out["lse_c"], out["S"], out["A"], out["KL"],
                   out["flags"], ws, entropy_d=out["H_d"], pd_x=out["pd_x"])
    torch.cuda.synchronize()
    return {n: (None if t is None else t.cpu().numpy()) for n, t in out.items()}


def gpu_accept_estimate(S, A, edges_s, edges_a, table):
    P = sv()
    S, A = dev(S, torch.float32), dev(A, torch.float32)
    p_hat = torch.empty_like(S)
    flag = torch.full(S.shape, 9, dtype=torch.uint8, device="cuda")
    P.sv_accept_estimate(S, A, dev(edges_s), dev(edges_a), dev(table), p_hat, flag)
    torch.cuda.synchronize()
    return p_hat.cpu().numpy(), flag.cpu().numpy()


def gpu_select_length(p_hat, latency, mode):
    P = sv()
    p_hat = dev(p_hat, torch.float32)
    B, k = p_hat.shape
    gamma = torch.full((B,), -9, dtype=torch.int32, device="cuda")
    offs = torch.full((B + 1,), -9, dtype=torch.int32, device="cuda")
    total = torch.full((1,), -9, dtype=torch.int32, device="cuda")
    P.sv_select_length(p_hat, dev(latency, torch.float32), mode, gamma, offs, total)
    torch.cuda.synchronize()
    return gamma.cpu().numpy(), offs.cpu().numpy(), int(total.item())


def gpu_verify(z_t, z_d, x, gamma=None, t_offsets=None, seed=0, step=0):
    P = sv()
    B, k, V = z_d.shape
    tokens = torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda")
    n_acc = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    flags = torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda")
    ratio = torch.full((B, k), -5.0, dtype=torch.float32, device="cuda")
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(z_d))
    g = None if gamma is None else dev(gamma, torch.int32)
    o = None if t_offsets is None else dev(t_offsets, torch.int32)
    P.sv_verify_sample(z_t, o, z_d, x, g, seed, step, tokens, n_acc, flags, ratio, ws)
    torch.cuda.synchronize()
    return dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
                flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())


def gpu_verify_chained(z_t, z_d, z_c, x, gamma=None, t_offsets=None, seed=0, step=0):
    """sv_row_stats, then sv_verify_sample_chained on the same workspace."""
    P = sv()
    B, k, V = z_d.shape
    mk = lambda: torch.full((B, k), -7.0, dtype=torch.float32, device="cuda")
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(z_d))
    P.sv_row_stats(z_d, z_c, x, mk(), mk(), mk(), mk(), None, None, ws)
    tokens = torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda")
    n_acc = torch.full((B,), -5, dtype=torch.int32, device="cuda")
    flags = torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda")
    ratio = torch.full((B, k), -5.0, dtype=torch.float32, device="cuda")
    g = None if gamma is None else dev(gamma, torch.int32)
    o = None if t_offsets is None else dev(t_offsets, torch.int32)
    P.sv_verify_sample_chained(z_t, o, z_d, x, g, seed, step, tokens, n_acc, flags, ratio, ws)
    torch.cuda.synchronize()
    fl = flags.cpu().numpy().astype(np.uint32)
    assert not (fl & P.binding.FLAG_NO_CHAIN).any(), "the chained call did not find the statistics pass"
    return dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(), flags=fl, ratio=ratio.cpu().numpy())


# ------------------------------------------------------------------ compare
def close(got, ref, rel=REL, abs_floor=0.0):
    """|got - ref| <= rel |ref| + abs_floor, NaN = NaN, inf = inf.  A float32
    result is compared with what float32 can hold of the reference: beyond its
    range the reference counts as inf, below its normal range as zero."""
    if np.asarray(got).dtype == np.float32:
        with np.errstate(over="ignore", under="ignore"):
            ref = np.asarray(ref, dtype=np.float64).astype(np.float32)
        abs_floor = max(abs_floor, float(np.finfo(np.float32).tiny))
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    both_nan = np.isnan(got) & np.isnan(ref)
    both_inf = np.isinf(got) & np.isinf(ref) & (np.sign(got) == np.sign(ref))
    with np.errstate(invalid="ignore"):
        ok = np.abs(got - ref) <= rel * np.abs(ref) + abs_floor
    return ok | both_nan | both_inf


def assert_row_stats(got, ref, with_kl=True):
    """fp32 stats within 1e-5 relative (S additionally to 2e-31 absolute: below that its terms
    underflow float32).  TV = 1 - S and KL are sums of
    probability differences whose entries carry ~1e-7 relative error each, so
    near zero they get an absolute floor: 2e-6 for KL and the entropy, 5e-6 for
    TV (on a flat row every term has the same exponent, near -17 at 1e5 entries,
    so the rounding of that exponent, up to 6.6e-7 relative, and of the equal
    additions no longer average out: 3.7e-6 has been observed)."""
    for name in ("lse_d", "lse_c"):
        ok = close(got[name], ref[name], REL, 1e-6)
        assert ok.all(), (name, got[name][~ok], ref[name][~ok])
    # (terms of S below 2^-126 underflow float32 on the HIP side: an S of that order of
    #  magnitude - disjoint distributions - is resolved to V * 2^-126 only; V <= 2^24)
    ok = close(got["S"], ref["S"], REL, float(2 ** 24 * np.finfo(np.float32).tiny))
    assert ok.all(), ("S", got["S"][~ok], ref["S"][~ok])
    ok = close(got["A"], ref["A"], REL, 1e-30)
    assert ok.all(), ("A", got["A"][~ok], ref["A"][~ok])
    tv = np.maximum(0, 1 - got["S"].astype(np.float64))
    ok = close(tv, ref["TV"], REL, 5e-6)
    assert ok.all(), ("TV", tv[~ok], ref["TV"][~ok])
    ok = close(got["pd_x"], ref["pd_x"], REL, 1e-37)
    assert ok.all(), ("pd_x", got["pd_x"][~ok], ref["pd_x"][~ok])
    if with_kl:
        ok = close(got["KL"], ref["KL"], REL, 2e-6)
        assert ok.all(), ("KL", got["KL"][~ok], ref["KL"][~ok])
        ok = close(got["H_d"], ref["H_d"], REL, 2e-6)
        assert ok.all(), ("H_d", got["H_d"][~ok], ref["H_d"][~ok])
    assert np.array_equal(got["flags"].astype(np.uint32), ref["flags"]), "flags"


def assert_verify(got, ref, k):
    """Token ids and accept counts bit-exact, except sequences where a near tie
    was flagged (either side): |u - ratio| < 1e-6 excludes the sequence; a
    sampling threshold within 1e-6 W + GPU_CDF_ABS_BAND of a CDF edge keeps the
    accept count exact and requires the token to be one of the admissible
    neighbours.  A residual whose exact mass lies within GPU_CDF_ABS_BAND of zero
    is below what fp32 probabilities resolve: either side may then have found it
    empty (FLAG_RESIDUAL_FALLBACK is not compared) and, if exactly one did, the
    token is only required to exist.  `ref` must come from oracle_verify.
    Returns the counts of near-tie and of near-edge / unresolved sequences."""
    B = got["tokens"].shape[0]
    n_tie = n_edge = 0
    for b in range(B):
        gf, rf = int(got["flags"][b]), int(ref["flags"][b])
        if (gf | rf) & O.FLAG_NEAR_TIE:
            n_tie += 1
            continue
        assert got["n_accept"][b] == ref["n_accept"][b], (b, got["n_accept"][b], ref["n_accept"][b])
        n = int(ref["n_accept"][b])
        assert np.array_equal(got["tokens"][b, :n], ref["tokens"][b, :n]), b
        assert np.all(got["tokens"][b, n + 1:] == -1), b
        hard = O.FLAG_BAD_ROW | O.FLAG_BAD_TOKEN | O.FLAG_RESIDUAL_FALLBACK
        unresolved = bool(ref["resid"][b] and ref["W"][b] <= GPU_CDF_ABS_BAND) or \
            bool((rf & O.FLAG_RESIDUAL_FALLBACK) and not (rf & O.FLAG_BAD_ROW))
        if unresolved:
            hard &= ~O.FLAG_RESIDUAL_FALLBACK
        assert (gf & hard) == (rf & hard), (b, gf, rf)
        ev = ~np.isnan(ref["ratio"][b])
        assert np.array_equal(np.isnan(got["ratio"][b]), ~ev), (b, got["ratio"][b], ref["ratio"][b])
        assert close(got["ratio"][b][ev], ref["ratio"][b][ev], REL, 1e-30).all(), \
            (b, got["ratio"][b], ref["ratio"][b])
        if unresolved and ((gf ^ rf) & O.FLAG_RESIDUAL_FALLBACK):
            n_edge += 1
            assert got["tokens"][b, n] >= 0, (b, got["tokens"][b])
        elif (gf | rf) & O.FLAG_NEAR_CDF_EDGE:
            n_edge += 1
            assert int(got["tokens"][b, n]) in set(int(t) for t in ref["admissible"][b]), \
                (b, got["tokens"][b, n], ref["admissible"][b])
        else:
            assert got["tokens"][b, n] == ref["tokens"][b, n], \
                (b, got["tokens"][b, n], ref["tokens"][b, n], ref["margin"][b], ref["W"][b])
    return n_tie, n_edge


def oracle_inputs(cfg):
    return dict(z_t=svgen.to_numpy_bits(cfg["z_t"]), z_d=svgen.to_numpy_bits(cfg["z_d"]),
                z_c=svgen.to_numpy_bits(cfg["z_c"]), x=cfg["x"].cpu().numpy())


def uniforms_of(seqs, k, seed=0, step=0):
    """The Philox uniforms (accept [n, k], sampling [n, k + 1]) of the sequences with batch
    indices `seqs`, for handing a slice of a batch to the oracle."""
    from oracle import philox
    seq = np.asarray(seqs)[:, None]
    ua, _ = philox.sv_uniforms(seed, step, np.broadcast_to(seq, (len(seqs), k)), np.arange(k)[None, :])
    _, us = philox.sv_uniforms(seed, step, np.broadcast_to(seq, (len(seqs), k + 1)), np.arange(k + 1)[None, :])
    return ua, us

