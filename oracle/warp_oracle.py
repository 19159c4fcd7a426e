"""Plain CPU oracle for the sampling warps applied to logits before the SV
computations: temperature, top-k and top-p (the sampling hyper-parameters the
SV paper lists per model series in its appendix table "Sampling
hyperparameters for each model series"), and the repetition penalty of the
same table, which acts on the logits before them and needs the token history.

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

Repetition penalty (the table gives one value per model series, not the
operation; the usual logits processor is used): every token that occurs in the
history of a position has its logit divided by theta if it is positive and
multiplied by theta otherwise, once per distinct token.  The history of drafted
position i of a sequence is the sequence's context plus the tokens drafted before
i.  The penalised logit is written back in the storage type, so the arithmetic
is fixed to keep both sides of the parity check on the same bits: theta and the
logit are float32, the product / quotient is the correctly rounded float32
operation, and bfloat16 storage rounds that to nearest-even.

Pins (tests/test_oracle_warp.py): torch.topk, a sort/cumsum rendering of top-p
on rows without ties, scipy soft-max for the temperature, minimality of the
kept set, monotonicity in K and P, whole-group treatment of ties; the three
warps in sequence and the repetition penalty against the logits processors of
the `transformers` package on rows without ties; the bfloat16 rounding against
torch's conversion.
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


def _store_like(values32, like):
    """float32 values in the storage type of `like`: float32 as is, uint16 = bfloat16 bit
    patterns rounded to nearest-even (NaN stays NaN)."""
    v = np.asarray(values32, dtype=np.float32)
    if np.asarray(like).dtype != np.uint16:
        return v
    u = v.view(np.uint32).astype(np.uint64)
    rounded = ((u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)).astype(np.uint16)
    nan = np.isnan(v)
    rounded[nan] = ((u[nan] >> np.uint64(16)) | np.uint64(0x0040)).astype(np.uint16)     # quiet, sign and payload top kept
    return rounded


def repetition_penalty(z, history, penalty, x=None):
    """Logits after the repetition penalty, in the storage type of `z`.

    z        [B, R, V] stored logits (float32, or uint16 bfloat16 bit patterns); row i of
             sequence b is position i
    history  [B, n_hist] context token ids, entries outside [0, V) (padding: -1) are ignored
    x        optional [B, k] drafted tokens: position i is also penalised for x[b, :min(i, k)]
    penalty  theta > 0, taken as a float32
    """
    z = np.asarray(z)
    out = z.copy()
    B, R, V = z.shape
    theta = np.float32(penalty)
    history = np.asarray(history)
    for b in range(B):
        for i in range(R):
            toks = list(history[b])
            if x is not None:
                toks += list(np.asarray(x)[b, :min(i, np.asarray(x).shape[1])])
            toks = sorted({int(t) for t in toks if 0 <= int(t) < V})          # once per distinct token
            if not toks:
                continue
            if z.dtype == np.uint16:
                vals = (z[b, i, toks].astype(np.uint32) << np.uint32(16)).view(np.float32)
            else:
                vals = z[b, i, toks].astype(np.float32)
            with np.errstate(all="ignore"):
                new = np.where(vals < 0, vals * theta, vals / theta).astype(np.float32)
            out[b, i, toks] = _store_like(new, z)
    return out

