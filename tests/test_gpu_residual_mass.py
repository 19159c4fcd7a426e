"""Residual draws at small residual mass W (target and draft nearly equal).

The speculative-sampling rule draws from the normalised residual max(0, P_t - P_d)
whatever its mass (Sec. 4.2, last paragraph, of the SV paper points to that rule; it has
no floor).  The oracle does so in fp64.  The HIP path holds probabilities in fp32, so
below W of about 1e-6 its residual is rounding noise, and at any W the edges of its CDF
are known only to about 5e-7 absolute.  These tests walk W from 0.15 down through that
limit and check the parity rule: off the flagged bands tokens are identical; on them the
token lies in the oracle's admissible set; where fp32 cannot tell the residual from an
empty one, the accept count still matches and a token is still produced."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O
import harness as H

pytestmark = pytest.mark.gpu


def _run(c, seed, step):
    z_t, z_d, x = c["z_t"].cuda(), c["z_d"].cuda(), c["x"].cuda()
    got = H.gpu_verify(z_t, z_d, x, seed=seed, step=step)
    ref = H.oracle_verify(svgen.to_numpy_bits(c["z_t"]), svgen.to_numpy_bits(c["z_d"]), c["x"].numpy(),
                          seed=seed, step=step)
    assert (ref["n_accept"] == 0).all()                      # the forced rejection
    n_tie, n_edge = H.assert_verify(got, ref, 1)
    assert n_tie == 0
    return got, ref, n_edge


def _report(tag, got, ref, n_edge):
    W = ref["W"]
    res = ref["resid"]
    exact = int(np.sum(((got["flags"] | ref["flags"]) & O.FLAG_NEAR_CDF_EDGE) == 0))
    lo = W[res].min() if res.any() else float("nan")
    hi = W[res].max() if res.any() else float("nan")
    print(f"\n  {tag}: {len(W)} sequences, residual mass {lo:.2e} .. {hi:.2e}, "
          f"{int((~res).sum())} without residual, tokens identical off the band {exact}, "
          f"inside the band (admissible) {n_edge}", flush=True)
    return exact


@pytest.mark.parametrize("dtype,lo,hi", [("f32", 1e-9, 0.5), ("bf16", 1e-5, 1.0)])
def test_residual_mass_walk(dtype, lo, hi):
    """V = 8192: the perturbation is walked over many decades, from a residual far above to
    one far below what fp32 resolves (and, in bf16, to rows that are equal: mass exactly 0)."""
    c = svgen.make_near_pairs(192, 8192, dtype, 77, lo, hi)
    got, ref, n_edge = _run(c, seed=5, step=1)
    W, res = ref["W"], ref["resid"]
    assert (W[res] < 1e-6).any() and (W[res] > 1e-3).any()
    if dtype == "bf16":
        assert (~res).any()                                  # equal rows: both sides fall back
        both = (~res) & ((ref["flags"] & O.FLAG_RESIDUAL_FALLBACK) != 0)
        assert ((got["flags"][both] & O.FLAG_RESIDUAL_FALLBACK) != 0).all()
    # a residual that fp32 does resolve is never reported as empty
    big = res & (W > 4 * H.GPU_CDF_ABS_BAND)
    assert ((got["flags"][big] & O.FLAG_RESIDUAL_FALLBACK) == 0).all()
    exact = _report(f"walk {dtype}", got, ref, n_edge)
    assert exact >= 20


@pytest.mark.parametrize("dtype,lo,hi,B", [("f32", 2e-5, 0.4, 384), ("bf16", 2e-3, 1.0, 384)])
def test_residual_mass_sweep_full_vocabulary(dtype, lo, hi, B):
    """V = 152064 (the headline vocabulary), residual mass from about 1e-5 to 0.15."""
    c = svgen.make_near_pairs(B, 152064, dtype, 78, lo, hi)
    got, ref, n_edge = _run(c, seed=6, step=2)
    W = ref["W"][ref["resid"]]
    assert W.min() < 1e-4 and W.max() > (1e-2 if dtype == "f32" else 2e-3)
    _report(f"sweep {dtype}", got, ref, n_edge)
