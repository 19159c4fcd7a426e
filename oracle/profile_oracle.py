"""Plain CPU oracle for building the acceptance profile P(T | S, A) and for the
information-gain figures of the SV paper (arxiv 2509.24328).

TEST INFRASTRUCTURE ONLY (see sv_oracle): float64 NumPy, sample by sample, no
code shared with the HIP path.

What follows the paper, by passage:

* profile table .......... appendix definition of the observed probability:
                           samples are grouped (binned) by the values of S and A
                           and the acceptance probability is averaged per cell
* X ...................... Sec. 4.1 / Sec. 7.3 "Information Gain from S and A":
                           X is the acceptance probability of a drafted token
                           in the target model under the speculative-sampling
                           rule, min(1, p_t(x) / p_d(x)), observed for every
                           drafted token (no verification-length optimisation)
* H(X), H(X|S,A), I ...... Sec. 4.1: I(X;Y) = H(X) - H(X|Y), with S and A
                           discretised into equal-sized sub-ranges or by the
                           "adaptive" binning that puts smaller bins where the
                           samples are denser (Sec. 7.3, Table 1)

Readings where the paper is silent:
* X is continuous; the paper never says how it is discretised for H(X) (its
  H(X) of 1.38-1.78 bits rules out the binary accept event).  Here: n_x
  equal-width bins on [0, 1], the top one closed, n_x chosen by the caller.
* "Adaptive" binning: equal-count (quantile) edges per axis on a product grid
  (16 x 17 gives the paper's 272 cells); interior edge j of n_bins is the
  floor(j n / n_bins)-th smallest sample, the outer edges are 0 and 1.
* Empty cells get the global mean acceptance probability.
* Samples with a NaN in S, A or X (bad rows, impossible tokens) are skipped.
Entropies are in bits.

Pins (tests/test_oracle_profile.py): numpy.histogramdd, scipy.stats.entropy,
closed forms (independent and deterministic X), per-cell means by masking,
equal-count property of the quantile edges.
"""
from __future__ import annotations

import numpy as np

from . import sv_oracle as O


def accept_probability_ratio(z_t, z_d, x):
    """p_t(x)/p_d(x) for every drafted position (b, i), i < k: no early stop.

    z_t: [B, >=k, V] (rows beyond k are ignored), z_d: [B, k, V], x: [B, k].
    Returns (ratio float64 [B, k], flags uint32 [B, k]); NaN for bad rows/tokens.
    """
    z_t = np.asarray(z_t)
    z_d = np.asarray(z_d)
    x = np.asarray(x)
    B, k, V = z_d.shape
    ratio = np.full((B, k), np.nan)
    flags = np.zeros((B, k), dtype=np.uint32)
    for b in range(B):
        for i in range(k):
            ratio[b, i], flags[b, i] = O.accept_ratio(z_t[b, i], z_d[b, i], int(x[b, i]))
    return ratio, flags


def x_bin(ratio, n_x):
    """Bin of X = clip(ratio, 0, 1) among n_x equal bins of [0, 1], top closed.
    Evaluated in float32 (clip, multiply by n_x, floor) so that both sides of a
    parity check take the same decision.  NaN -> -1."""
    r = np.float32(ratio)
    if np.isnan(r):
        return -1
    xc = np.float32(min(np.float32(1.0), max(np.float32(0.0), r)))
    return int(min(n_x - 1, int(np.floor(np.float32(xc * np.float32(n_x))))))


def accumulate(S, A, ratio, edges_s, edges_a, n_x, counts=None, sum_x=None):
    """Add samples to the joint histogram counts[n_s, n_a, n_x] (int64) and to the
    per-cell sums of X, sum_x[n_s, n_a] (float64).  Cells use the same bin rule
    as the estimate lookup (half-open bins, top closed, clamped)."""
    S = np.asarray(S, dtype=np.float32).ravel()
    A = np.asarray(A, dtype=np.float32).ravel()
    ratio = np.asarray(ratio, dtype=np.float32).ravel()
    edges_s = np.asarray(edges_s, dtype=np.float32)
    edges_a = np.asarray(edges_a, dtype=np.float32)
    n_s, n_a = len(edges_s) - 1, len(edges_a) - 1
    if counts is None:
        counts = np.zeros((n_s, n_a, n_x), dtype=np.int64)
        sum_x = np.zeros((n_s, n_a), dtype=np.float64)
    for j in range(S.size):
        if np.isnan(S[j]) or np.isnan(A[j]) or np.isnan(ratio[j]):
            continue
        i_s = O._bin_index(S[j], edges_s)
        i_a = O._bin_index(A[j], edges_a)
        xc = np.float32(min(np.float32(1.0), max(np.float32(0.0), ratio[j])))
        counts[i_s, i_a, x_bin(ratio[j], n_x)] += 1
        sum_x[i_s, i_a] += float(xc)
    return counts, sum_x


def entropy_bits(p):
    p = np.asarray(p, dtype=np.float64)
    p = p[p > 0]
    return float(-(p * np.log2(p)).sum())


def finalize(counts, sum_x):
    """Profile table and information figures from the accumulated histogram.

    table[n_s, n_a] float32: mean X of the cell; empty cells: the global mean;
    no samples at all: 0.  info = (H(X), H(X | S,A), I(X; S,A)) in bits.
    """
    counts = np.asarray(counts, dtype=np.float64)
    sum_x = np.asarray(sum_x, dtype=np.float64)
    cell_n = counts.sum(axis=2)
    N = cell_n.sum()
    table = np.zeros(cell_n.shape, dtype=np.float64)
    if N > 0:
        glob = sum_x.sum() / N
        for idx in np.ndindex(cell_n.shape):
            table[idx] = sum_x[idx] / cell_n[idx] if cell_n[idx] > 0 else glob
        h_x = entropy_bits(counts.sum(axis=(0, 1)) / N)
        h_cond = 0.0
        for idx in np.ndindex(cell_n.shape):
            if cell_n[idx] > 0:
                h_cond += cell_n[idx] / N * entropy_bits(counts[idx] / cell_n[idx])
    else:
        h_x = h_cond = 0.0
    return table.astype(np.float32), (h_x, h_cond, h_x - h_cond)


def quantile_edges(values, n_bins, lo=0.0, hi=1.0):
    """Equal-count edges: [lo, q_1, ..., q_{n_bins-1}, hi], q_j = the
    floor(j n / n_bins)-th smallest of the n non-NaN samples (0-based)."""
    v = np.asarray(values, dtype=np.float32).ravel()
    v = np.sort(v[~np.isnan(v)])
    n = v.size
    edges = np.empty(n_bins + 1, dtype=np.float32)
    edges[0], edges[n_bins] = np.float32(lo), np.float32(hi)
    for j in range(1, n_bins):
        edges[j] = v[(j * n) // n_bins] if n > 0 else np.float32(lo)
    return edges
