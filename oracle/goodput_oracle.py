"""Plain CPU oracle for the step-level comparison of acceptance estimators and
for the goodput bookkeeping of the SV paper (arxiv 2509.24328).

TEST INFRASTRUCTURE ONLY (see sv_oracle): float64 NumPy on top of sv_oracle and
profile_oracle, no code shared with the HIP path.

What follows the paper, by passage:

* estimators ........ Sec. 2 "Predicting Speculation Accuracy" names two families
                      of prior predictors: the draft model's probability of its
                      own sampled token (Tetris, DySpec) and the entropy of the
                      draft distribution (SVIP, AdaEDL, DISCO).  Sec. 4 replaces
                      them by the pair (S, A) of the companion model.  Sec. 7.3
                      compares signals by the information they carry about the
                      acceptance probability X.
* estimate .......... appendix definition of the observed probability: the mean
                      acceptance probability of the profiled samples that fall
                      into the same cell as the signal.  The same definition is
                      applied to every signal here, so that the estimators differ
                      in their signal only: (S, A) on a 2-D grid, the draft
                      entropy H(P_d) on a 1-D grid, P_d(x) on a 1-D grid, each
                      with the same number of cells.
* lengths, goodput .. Sec. 5: batch-greedy lengths from the estimates and the
                      latency profile; goodput = accepted tokens per unit of
                      (profiled) verification latency.  Plain speculative
                      decoding ("sd") verifies all k drafted tokens.

Readings where the paper is silent: how the prior predictors turn their signal
into a probability differs from paper to paper (thresholds, fitted bounds); the
profiled-mean rule above is the one form that needs no extra parameters and is
the best any calibrated function of the signal can do on the profiled samples.
The 1-D grids use equal-count edges (the paper's "adaptive" binning), the (S, A)
grid uniform edges.  Goodput counts accepted drafted tokens only, as the paper's
formula does (no +1 for the token every step emits anyway).
"""
from __future__ import annotations

import numpy as np

from . import profile_oracle as PO
from . import sv_oracle as O

ESTIMATORS = ("sv", "entropy", "probability")
UNIT_EDGES = np.array([0.0, 1.0], dtype=np.float32)


def signals(z_d, z_c, x):
    """The per-position signals of the three estimators, float32 [B, k] each:
    (S, A), the draft entropy H(P_d) in nats, the draft's probability P_d(x)."""
    r = O.row_stats(z_d, z_c, x)
    f = lambda a: np.asarray(a, dtype=np.float32)
    return dict(S=f(r["S"]), A=f(r["A"]), H_d=f(r["H_d"]), pd_x=f(r["pd_x"]))


def axes_of(name, sig):
    """(first-axis values, second-axis values) an estimator looks its table up with."""
    if name == "sv":
        return sig["S"], sig["A"]
    zero = np.zeros_like(sig["S"])
    if name == "entropy":
        return sig["H_d"], zero
    if name == "probability":
        return sig["pd_x"], zero
    raise ValueError(name)


def build_profile(name, sig, ratio, V, cells=100, n_x=10):
    """Profile of one estimator from held-out samples: (edges_1, edges_2, table, info).

    sv: sqrt(cells) x sqrt(cells) uniform edges on [0,1]^2; entropy: `cells` equal-count
    edges on [0, ln V]; probability: `cells` equal-count edges on [0, 1]; second axis of
    the 1-D estimators: the single bin [0, 1].  info = (H(X), H(X|signal), gain) in bits.
    """
    a1, a2 = axes_of(name, sig)
    if name == "sv":
        n = int(round(np.sqrt(cells)))
        e1 = np.linspace(0.0, 1.0, n + 1).astype(np.float32)
        e2 = e1.copy()
    else:
        hi = float(np.float32(np.log(V))) if name == "entropy" else 1.0
        e1 = PO.quantile_edges(a1, cells, 0.0, hi)
        e2 = UNIT_EDGES
    counts, sum_x = PO.accumulate(a1, a2, ratio, e1, e2, n_x)
    table, info = PO.finalize(counts, sum_x)
    return e1, e2, table, info


def estimate(name, sig, profile):
    """p_hat [B, k] float32 and the edge flags of one estimator."""
    a1, a2 = axes_of(name, sig)
    e1, e2, table = profile[:3]
    return O.accept_estimate(a1, a2, e1, e2, table)


def step(z_t, z_d, z_c, x, profiles, latency, seed, step_index):
    """One decode step under plain SD and under every estimator in `profiles`.

    Returns {name: dict(gamma [B], M, n_accept [B], accepted, verified, latency,
    near_edge (any lookup within the bin-edge band), near_tie [B] bool)} with name "sd"
    for plain speculative decoding.  The same Philox step serves all of them, as one
    serving step would: only the verified lengths differ.
    """
    B, k, _ = np.asarray(z_d).shape
    sig = signals(z_d, z_c, x)
    out = {}
    full = np.full(B, k, dtype=np.int32)
    plans = {"sd": (full, B * k, False)}
    for name in profiles:
        p_hat, edge = estimate(name, sig, profiles[name])
        g, _, M = O.select_length(p_hat, latency)
        plans[name] = (g, M, bool(edge.any()))
    for name, (g, M, near_edge) in plans.items():
        v = O.verify_sample(z_t, z_d, x, gamma=g, seed=seed, step=step_index)
        out[name] = dict(gamma=g, M=int(M), n_accept=v["n_accept"], accepted=int(v["n_accept"].sum()),
                         verified=int(M), latency=float(latency[M]), near_edge=near_edge,
                         near_tie=(v["flags"] & O.FLAG_NEAR_TIE) != 0)
    return out, sig


def totals(per_step):
    """Goodput bookkeeping over a run: per_step = list of step() results."""
    res = {}
    for name in per_step[0]:
        acc = sum(s[name]["accepted"] for s in per_step)
        ver = sum(s[name]["verified"] for s in per_step)
        lat = sum(s[name]["latency"] for s in per_step)
        B = per_step[0][name]["gamma"].shape[0]
        res[name] = dict(accepted=acc, verified=ver, latency=lat,
                         goodput=acc / lat if lat else 0.0,
                         accept_rate=acc / ver if ver else 0.0,
                         mean_verified_per_seq=ver / (len(per_step) * B))
    return res
