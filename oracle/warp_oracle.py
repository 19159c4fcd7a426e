"""Plain CPU oracle for the sampling warps applied to logits before the SV
computations: temperature, top-k and top-p (the sampling hyper-parameters the
SV paper lists per model series in its appendix table "Sampling
hyperparameters for each model series"; repetition penalty needs the token
history and is not covered).

TEST INFRASTRUCTURE ONLY (see sv_oracle): float64 NumPy, one row at a time.

The paper only lists the values; the operations are the usual logits
processors, applied in the usual order temperature -> top-k -> top-p:

  y_v = z_v / T
  top-k:  keep the entries whose value is at least the K-th largest value
  top-p:  over the entries kept so far, with p = softmax(y), walk the distinct
          values downwards and keep whole groups of equal value until the kept
          mass reaches P; the value of the last group kept is the cutoff
  warped row:  y_v if z_v >= cutoff else -inf

Reading on ties: entries of equal value are kept or dropped together (with
bfloat16 logits equal values are common, and any finer rule would depend on an
arbitrary sort order).  Without ties this is exactly "the K most likely
tokens" and "the smallest set of most likely tokens whose mass reaches P".
K <= 0 or K >= V switches top-k off, P >= 1 switches top-p off.

Pins (tests/test_oracle_warp.py): torch.topk, a sort/cumsum rendering of top-p
on rows without ties, scipy soft-max for the temperature, minimality of the
kept set, monotonicity in K and P, whole-group treatment of ties.
"""
from __future__ import annotations

import numpy as np

from . import sv_oracle as O

NEAR_TIE_EPS = 1e-6


def warp_cutoff(row, temperature=1.0, top_k=0, top_p=1.0):
    """Cutoff value of one row (in raw logit units) and flag bits.

    Returns (cutoff, flags): entries with z >= cutoff are kept; -inf keeps all.
    Bad rows (NaN, +inf, no finite entry) give (nan, FLAG_BAD_ROW).
    FLAG_NEAR_TIE marks a top-p decision within 1e-6 of P.
    """
    z = O.upcast(row)
    V = z.shape[0]
    m = np.max(z) if V else -np.inf
    if V == 0 or np.isnan(m) or np.isinf(m):
        return np.nan, O.FLAG_BAD_ROW
    cutoff, flags = -np.inf, 0
    if 0 < top_k < V:
        cutoff = np.partition(z, V - top_k)[V - top_k]          # K-th largest value
    if top_p < 1.0:
        kept = z[z >= cutoff]
        y = kept / float(temperature)
        w = np.exp(y - y.max())
        total = w.sum()
        vals = np.unique(kept)[::-1]                              # distinct values, descending
        acc = 0.0
        for v in vals:
            acc += w[kept == v].sum()
            frac = acc / total
            if abs(frac - top_p) < NEAR_TIE_EPS:
                flags |= O.FLAG_NEAR_TIE
            if frac >= top_p:
                cutoff = max(cutoff, v)
                break
    return float(cutoff), flags


def warp_rows(z, temperature=1.0, top_k=0, top_p=1.0):
    """Warp every row of z [..., V]: float64 array of z/T with the dropped
    entries at -inf, the per-row cutoffs and flags.  Bad rows pass through
    unchanged (divided by T) so that the downstream oracle flags them itself."""
    z = np.asarray(z)
    lead = z.shape[:-1]
    out = np.empty(z.shape, dtype=np.float64)
    cut = np.empty(lead, dtype=np.float64)
    flags = np.zeros(lead, dtype=np.uint32)
    for idx in np.ndindex(lead):
        row = O.upcast(z[idx])
        c, f = warp_cutoff(z[idx], temperature, top_k, top_p)
        cut[idx], flags[idx] = c, f
        y = row / float(temperature)
        if not np.isnan(c):
            y = np.where(row >= c, y, -np.inf)
        out[idx] = y
    return out, cut, flags
