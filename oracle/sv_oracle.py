"""Plain CPU oracle for the Speculative Verification (SV) decode-step hot path.

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct
definition the HIP kernels are checked against.  Only tests, the smoke check
and the CPU-baseline leg of the benchmark may import it.  It shares no code,
tables or helpers with the HIP path and never imports it.

Everything is float64 after an exact upcast of the stored inputs (float32, or
bfloat16 carried as uint16 bit patterns), one row at a time, with no blocking,
fusion or reordering beyond what the definitions state.

What follows the paper (arxiv 2509.24328), by passage:

* indicators S and A ........ Sec. 4.2 "Indicators in Companion Model" and the
                              two definitions opening Appendix "Optimality of
                              SV's Verification Length Selection"
* estimate P^(T_i | S, A) ... binned-profile definition in the same appendix
* P_gamma(N), E(N | gamma) .. Sec. 5 "Scheduling for Speculative Verification"
                              (the P_gamma(N) equation) and its appendix
                              definition
* goodput, gamma search ..... Sec. 5 (incremental search, batch greedy rule)
                              and the goodput definition in the appendix
* verification .............. Sec. 4.2, last paragraph: forwarded tokens go
                              through the standard speculative-sampling rule
                              (Leviathan et al.), dropped positions are drawn
                              by the target from its own distribution

The paper cites the speculative-sampling rule without restating it; the rule
used here is the standard one: accept drafted token x with probability
min(1, p_t(x)/p_d(x)); on the first rejection draw from the normalised
residual max(0, p_t - p_d); if every verified token is accepted draw one more
token from the target distribution of the next position.

Pins (tests/test_oracle_*.py, all CPU): scipy/torch log-sum-exp, V=2 closed
form of S, E_{x~P_d}[A] = S, acceptance probability = 1 - TV, per-position and
whole-step enumeration on tiny vocabularies for every gamma, sum_N P_gamma(N)
= 1, E(N|gamma) = sum of prefix products, brute-force optimality of the greedy
selection, first-peak == argmax on latency tables obeying the paper's latency
assumption, numpy.searchsorted for the inverse CDF.  No function here is
"parity unpinned"; the numbers in the paper's own tables need its trained
models and are not reproduced.
"""
from __future__ import annotations

import numpy as np

from . import philox

# Per-sequence / per-row condition bits (data-dependent, never errors).
FLAG_BAD_ROW = 1            # a row with a NaN or no finite entry was needed
FLAG_NEAR_TIE = 2           # |u - min(1, rho)| < NEAR_TIE_EPS at an evaluated position
FLAG_RESIDUAL_FALLBACK = 4  # residual mass exactly 0 / non-finite, or bad draft row; target row used instead
FLAG_NEAR_CDF_EDGE = 8      # sampling threshold within CDF_EDGE_EPS * W of a CDF edge
FLAG_BAD_TOKEN = 16         # drafted token id outside [0, V)

NEAR_TIE_EPS = 1e-6
CDF_EDGE_EPS = 1e-6
BIN_EDGE_EPS = np.float32(1e-5)

MODE_BATCH_GREEDY = 0
MODE_PER_SEQUENCE = 1


# ----------------------------------------------------------------------------
# inputs
# ----------------------------------------------------------------------------
def upcast(z):
    """Exact conversion of stored logits to float64.

    uint16 arrays are bfloat16 bit patterns (the upper half of a float32).
    """
    z = np.asarray(z)
    if z.dtype == np.uint16:
        return (z.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if z.dtype in (np.float32, np.float64):
        return z.astype(np.float64)
    raise TypeError(f"unsupported logit dtype {z.dtype}")


# ----------------------------------------------------------------------------
# row normalisers
# ----------------------------------------------------------------------------
def log_softmax_row(z):
    """(LSE, log p) of one row of logits, float64.

    LSE = m + log sum_v exp(z_v - m) with m = max_v z_v.  -inf entries carry
    zero mass.  A row holding a NaN or +inf, or no finite entry at all, is
    'bad': LSE and every log p are NaN.
    """
    z = np.asarray(z, dtype=np.float64)
    m = np.max(z) if z.size else -np.inf
    if z.size == 0 or np.isnan(m) or np.isinf(m):
        return np.nan, np.full(z.shape, np.nan)
    s = np.sum(np.exp(z - m))
    lse = m + np.log(s)
    return lse, z - lse


# ----------------------------------------------------------------------------
# a1/a2: S, A and divergences between draft and companion
# ----------------------------------------------------------------------------
def row_stats(z_d, z_c, x):
    """Draft/companion indicators for every (sequence, position).

    z_d, z_c: [B, k, V] stored logits; x: [B, k] drafted token ids.
    Returns a dict of [B, k] arrays:
      lse_d, lse_c : row log-sum-exp
      S            : sum_v min(P_d(v), P_c(v))
      A            : min(1, P_c(x) / P_d(x)), evaluated in log space
      TV           : max(0, 1 - S)
      KL           : sum_{v: P_d(v) > 0} P_d(v) (log P_d(v) - log P_c(v))
      H_d          : draft entropy -sum_{v: P_d(v) > 0} P_d(v) log P_d(v), nats
      pd_x         : P_d(x), the draft's probability of its own drafted token
      flags        : FLAG_BAD_ROW / FLAG_BAD_TOKEN bits (uint32)
    If P_d(x) = 0 the ratio is taken as saturated, A = 1.
    """
    z_d = np.asarray(z_d)
    z_c = np.asarray(z_c)
    x = np.asarray(x)
    B, k, V = z_d.shape
    out = {n: np.full((B, k), np.nan) for n in ("lse_d", "lse_c", "S", "A", "TV", "KL", "H_d", "pd_x")}
    flags = np.zeros((B, k), dtype=np.uint32)
    for b in range(B):
        for i in range(k):
            lse_d, lp_d = log_softmax_row(upcast(z_d[b, i]))
            lse_c, lp_c = log_softmax_row(upcast(z_c[b, i]))
            out["lse_d"][b, i] = lse_d
            out["lse_c"][b, i] = lse_c
            if np.isnan(lse_d) or np.isnan(lse_c):
                flags[b, i] |= FLAG_BAD_ROW
                continue
            p_d = np.exp(lp_d)
            p_c = np.exp(lp_c)
            S = np.sum(np.minimum(p_d, p_c))
            out["S"][b, i] = S
            out["TV"][b, i] = max(0.0, 1.0 - S)
            pos = p_d > 0
            with np.errstate(invalid="ignore"):
                out["KL"][b, i] = np.sum(p_d[pos] * (lp_d[pos] - lp_c[pos]))
            out["H_d"][b, i] = -np.sum(p_d[pos] * lp_d[pos])
            t = int(x[b, i])
            if t < 0 or t >= V:
                flags[b, i] |= FLAG_BAD_TOKEN
                continue
            out["pd_x"][b, i] = p_d[t]
            if lp_d[t] == -np.inf:
                out["A"][b, i] = 1.0
            else:
                out["A"][b, i] = min(1.0, float(np.exp(lp_c[t] - lp_d[t])))
    out["flags"] = flags
    return out


# ----------------------------------------------------------------------------
# a3: binned acceptance estimate
# ----------------------------------------------------------------------------
def _bin_index(v, edges):
    """Half-open bins [e_j, e_{j+1}) over ascending edges e_0..e_n, the top bin
    closed, values outside clamped into the first/last bin.  NaN -> bin 0."""
    n = len(edges) - 1
    if np.isnan(v):
        return 0
    idx = 0
    for j in range(1, n + 1):
        if edges[j] <= v:
            idx = j
    return min(max(idx, 0), n - 1)


def _near_edge(v, edges):
    """True when float32 |v - e_j| <= 1e-5 for an interior edge j (the only
    edges at which the bin decision changes), or v is NaN.  Evaluated in
    float32 so that both sides of a parity check take the same decision."""
    v = np.float32(v)
    if np.isnan(v):
        return True
    for e in np.asarray(edges, dtype=np.float32)[1:-1]:
        if np.abs(np.float32(v - e)) <= BIN_EDGE_EPS:
            return True
    return False


def accept_estimate(S, A, edges_s, edges_a, table):
    """p_hat = table[bin_s(S), bin_a(A)] for float32 S, A of any shape.

    edges_s: n_s + 1 ascending float32 edges, edges_a: n_a + 1, table
    [n_s, n_a] float32: the mean observed acceptance probability of each
    (S, A) cell.  The full product grid is used; one table serves every
    position.  Returns (p_hat float32, edge_flag uint8).
    """
    S = np.asarray(S, dtype=np.float32)
    A = np.asarray(A, dtype=np.float32)
    edges_s = np.asarray(edges_s, dtype=np.float32)
    edges_a = np.asarray(edges_a, dtype=np.float32)
    table = np.asarray(table, dtype=np.float32)
    p_hat = np.empty(S.shape, dtype=np.float32)
    flag = np.zeros(S.shape, dtype=np.uint8)
    for idx in np.ndindex(S.shape):
        i_s = _bin_index(S[idx], edges_s)
        i_a = _bin_index(A[idx], edges_a)
        p_hat[idx] = table[i_s, i_a]
        flag[idx] = 1 if (_near_edge(S[idx], edges_s) or _near_edge(A[idx], edges_a)) else 0
    return p_hat, flag


# ----------------------------------------------------------------------------
# a4: distribution and expectation of the accepted count
# ----------------------------------------------------------------------------
def sanitize_p(p_hat):
    """Estimates as probabilities: clamp to [0, 1], NaN -> 0 (float64)."""
    p = np.asarray(p_hat, dtype=np.float64).copy()
    p[np.isnan(p)] = 0.0
    return np.clip(p, 0.0, 1.0)


def p_gamma(p, gamma):
    """P_gamma(N = 0..gamma) for one sequence with acceptance estimates p[0..k).

    N < gamma : (1 - p_{N+1}) * prod_{i<=N} p_i ;  N = gamma : prod_{i<=gamma} p_i.
    """
    p = sanitize_p(p)
    out = np.zeros(gamma + 1)
    for n in range(gamma + 1):
        prod = 1.0
        for i in range(n):
            prod *= p[i]
        out[n] = prod * (1.0 - p[n]) if n < gamma else prod
    return out


def expected_accepted(p, gamma):
    """E(N | gamma) = sum_{i=1..gamma} i * P_gamma(N = i), as the paper defines it."""
    pg = p_gamma(p, gamma)
    return float(sum(i * pg[i] for i in range(1, gamma + 1)))


def prefix_products(p_hat):
    """c[b, j] = prod_{i<=j} p[b, i], accumulated left to right in float64.

    By P_gamma(N >= j) = c_j the expectation above equals sum_{j<=gamma} c_j,
    so c[b, gamma] is the gain in expected accepted length from verifying one
    more token of sequence b (pinned in the tests).
    """
    p = sanitize_p(p_hat)
    c = np.empty_like(p)
    for b in range(p.shape[0]):
        acc = 1.0
        for j in range(p.shape[1]):
            acc = acc * p[b, j]
            c[b, j] = acc
    return c


# ----------------------------------------------------------------------------
# a5: verification-length selection
# ----------------------------------------------------------------------------
def _greedy(c, latency):
    """Goodput-greedy selection over the sequences in c ([B', k]).

    Start from nothing; repeatedly take the not-yet-selected next token of the
    sequence whose gain c[b, gamma_b] is largest (ties: lowest b); keep it
    only while estimated goodput E_M / latency[M] strictly improves; stop at
    the first non-improvement.  E_M is accumulated in selection order.
    """
    Bp, k = c.shape
    gamma = np.zeros(Bp, dtype=np.int32)
    E = 0.0
    M = 0
    best = 0.0           # goodput of the empty selection
    while M < Bp * k:
        cand_b, cand_gain = -1, -1.0
        for b in range(Bp):
            if gamma[b] < k and c[b, gamma[b]] > cand_gain:
                cand_b, cand_gain = b, c[b, gamma[b]]
        E_new = E + cand_gain
        g_new = E_new / float(latency[M + 1])
        if not (g_new > best):
            break
        gamma[cand_b] += 1
        E, M, best = E_new, M + 1, g_new
    return gamma, M


def select_length(p_hat, latency, mode=MODE_BATCH_GREEDY):
    """Verification length per sequence from acceptance estimates p_hat [B, k].

    latency[M]: profiled latency of verifying M drafted tokens in total
    (batch mode: M = 0..B*k; per-sequence mode: M = 0..k), float32 > 0.
    Returns (gamma int32 [B], t_offsets int32 [B+1] = exclusive scan of
    gamma_b + 1, total_M).
    """
    p_hat = np.asarray(p_hat, dtype=np.float32)
    latency = np.asarray(latency, dtype=np.float32).astype(np.float64)
    B, k = p_hat.shape
    c = prefix_products(p_hat)
    if mode == MODE_BATCH_GREEDY:
        assert latency.size >= B * k + 1
        gamma, M = _greedy(c, latency)
    elif mode == MODE_PER_SEQUENCE:
        assert latency.size >= k + 1
        gamma = np.zeros(B, dtype=np.int32)
        for b in range(B):
            g, _ = _greedy(c[b:b + 1], latency)
            gamma[b] = g[0]
        M = int(gamma.sum())
    else:
        raise ValueError("mode")
    t_offsets = np.zeros(B + 1, dtype=np.int32)
    for b in range(B):
        t_offsets[b + 1] = t_offsets[b] + gamma[b] + 1
    return gamma.astype(np.int32), t_offsets, int(M)


# ----------------------------------------------------------------------------
# a6-a8: speculative-sampling verification
# ----------------------------------------------------------------------------
def accept_ratio(z_t_row, z_d_row, token):
    """rho = p_t(token) / p_d(token) in log space; NaN for bad rows/tokens.

    Returns (rho, flag_bits).  p_d(token) = 0 with p_t(token) > 0 gives +inf
    (always accepted); 0/0 gives NaN (rejected).
    """
    zt = upcast(z_t_row)
    zd = upcast(z_d_row)
    V = zt.shape[0]
    if token < 0 or token >= V:
        return np.nan, FLAG_BAD_TOKEN
    lse_t, _ = log_softmax_row(zt)
    lse_d, _ = log_softmax_row(zd)
    if np.isnan(lse_t) or np.isnan(lse_d):
        return np.nan, FLAG_BAD_ROW
    with np.errstate(invalid="ignore", over="ignore"):
        rho = np.exp((zt[token] - lse_t) - (zd[token] - lse_d))
    return float(rho), 0


def sampling_weights(z_t_row, z_d_row=None):
    """Unnormalised sampling weights w over the vocabulary and their mass W.

    With a draft row: the residual max(0, P_t - P_d), for any mass W > 0
    however small (the speculative-sampling rule has no floor, and float64 has
    no resolution limit that would call for one).  Without: P_t itself (bonus
    token / position the target generates on its own).  Only a residual of
    mass exactly 0 (P_t = P_d; a rejection can still happen there when the
    drafted token has no mass under either model), a non-finite one, or a bad
    draft row falls back to P_t.  Returns (w, W, flag_bits); a bad target row
    gives (None, nan, FLAG_BAD_ROW).
    """
    lse_t, lp_t = log_softmax_row(upcast(z_t_row))
    if np.isnan(lse_t):
        return None, np.nan, FLAG_BAD_ROW
    p_t = np.exp(lp_t)
    flags = 0
    if z_d_row is not None:
        lse_d, lp_d = log_softmax_row(upcast(z_d_row))
        if not np.isnan(lse_d):
            w = np.maximum(0.0, p_t - np.exp(lp_d))
            W = float(np.sum(w))
            if np.isfinite(W) and W > 0.0:
                return w, W, flags
        else:
            flags |= FLAG_BAD_ROW
        flags |= FLAG_RESIDUAL_FALLBACK
    return p_t, float(np.sum(p_t)), flags


def sampling_support(z_t_row):
    """Tokens the target gives any probability at all (P_t > 0)."""
    _, lp_t = log_softmax_row(upcast(z_t_row))
    return np.exp(lp_t) > 0


def inverse_cdf(w, W, u, abs_band=0.0, support=None):
    """Token = smallest v with cumsum(w)[v] > u * W; if rounding leaves none,
    the largest v with w_v > 0.

    Returns (token, margin, admissible) where margin = distance of the
    threshold to the nearer end of the token's CDF interval, divided by W, and
    admissible = ids of the tokens whose CDF interval meets
    [tau - h, tau + h], h = CDF_EDGE_EPS * W + abs_band.

    abs_band and support serve the comparison with an implementation whose
    cumulative sums carry an absolute error of up to abs_band (probabilities
    held in a narrower type): they change neither the token nor the margin.
    With abs_band = 0 only tokens of positive weight are admissible; with
    abs_band > 0 every token of `support` is (a weight that is 0 here can be a
    rounding-sized positive number there), support = None meaning w > 0.
    """
    cdf = np.cumsum(w)
    tau = u * W
    above = np.nonzero(cdf > tau)[0]
    if above.size:
        y = int(above[0])
    else:
        y = int(np.nonzero(w > 0)[0][-1])
    lo = cdf[y - 1] if y > 0 else 0.0
    margin = min(cdf[y] - tau, tau - lo) / W
    h = CDF_EDGE_EPS * W + abs_band
    prev = np.concatenate(([0.0], cdf[:-1]))
    can = (w > 0) if (support is None or abs_band == 0.0) else ((w > 0) | np.asarray(support))
    adm = np.nonzero(can & (cdf >= tau - h) & (prev <= tau + h))[0]
    return y, float(margin), adm.astype(np.int64)


def verify_sample(z_t, z_d, x, gamma=None, t_offsets=None, seed=0, step=0, uniforms=None,
                  cdf_abs_band=0.0):
    """One speculative-sampling verification step for B sequences.

    z_t : dense [B, k+1, V], or packed [sum_b (gamma_b + 1), V] with
          t_offsets [B+1] (row t_offsets[b] + i = target row of position i)
    z_d : [B, k, V];  x : [B, k] drafted tokens
    gamma : [B] verification lengths in 0..k (None: all k)
    uniforms : optional (u_accept [B, k], u_sample [B, k+1]) replacing the
          Philox stream (used by enumeration tests)
    cdf_abs_band : comparison aid, see inverse_cdf: widens FLAG_NEAR_CDF_EDGE
          and the admissible sets by an absolute band; tokens, accept counts
          and every other output are unaffected
    Returns dict: tokens int32 [B, k+1] (-1 padded), n_accept int32 [B],
    flags uint32 [B], ratio float64 [B, k] (NaN where not evaluated),
    margin float64 [B], admissible (list of arrays), W float64 [B] (mass of
    the weights drawn from), resid bool [B] (drawn from a residual),
    sample_row int32 [B].
    """
    z_t = np.asarray(z_t)
    z_d = np.asarray(z_d)
    x = np.asarray(x)
    B, k, V = z_d.shape
    if gamma is None:
        gamma = np.full(B, k, dtype=np.int32)
    gamma = np.asarray(gamma)

    def t_row(b, i):
        if t_offsets is None:
            return z_t[b, i]
        assert i <= gamma[b]
        return z_t[int(t_offsets[b]) + i]

    tokens = np.full((B, k + 1), -1, dtype=np.int32)
    n_accept = np.zeros(B, dtype=np.int32)
    flags = np.zeros(B, dtype=np.uint32)
    ratio = np.full((B, k), np.nan)
    margin = np.full(B, np.nan)
    Wout = np.full(B, np.nan)
    sample_row = np.zeros(B, dtype=np.int32)
    resid = np.zeros(B, dtype=bool)
    admissible = []
    for b in range(B):
        g = int(gamma[b])
        assert 0 <= g <= k
        n = 0
        for i in range(g):
            rho, fl = accept_ratio(t_row(b, i), z_d[b, i], int(x[b, i]))
            flags[b] |= fl
            ratio[b, i] = rho
            if uniforms is None:
                u, _ = philox.sv_uniforms(seed, step, b, i)
                u = float(u)
            else:
                u = float(uniforms[0][b, i])
            if not np.isnan(rho) and abs(u - min(1.0, rho)) < NEAR_TIE_EPS:
                flags[b] |= FLAG_NEAR_TIE
            if u < rho:          # False for NaN
                n += 1
            else:
                break
        n_accept[b] = n
        sample_row[b] = n
        tokens[b, :n] = x[b, :n]
        if uniforms is None:
            _, up = philox.sv_uniforms(seed, step, b, n)
            up = float(up)
        else:
            up = float(uniforms[1][b, n])
        w, W, fl = sampling_weights(t_row(b, n), z_d[b, n] if n < g else None)
        flags[b] |= fl
        Wout[b] = W
        if w is None:
            admissible.append(np.zeros(0, dtype=np.int64))
            continue            # bad target row: no token can be drawn, stays -1
        resid[b] = n < g and not (fl & FLAG_RESIDUAL_FALLBACK)
        support = sampling_support(t_row(b, n)) if cdf_abs_band > 0.0 else None
        y, mg, adm = inverse_cdf(w, W, up, cdf_abs_band, support)
        tokens[b, n] = y
        margin[b] = mg
        admissible.append(adm)
        if mg * W < CDF_EDGE_EPS * W + cdf_abs_band:
            flags[b] |= FLAG_NEAR_CDF_EDGE
    return dict(tokens=tokens, n_accept=n_accept, flags=flags, ratio=ratio, margin=margin,
                admissible=admissible, W=Wout, resid=resid, sample_row=sample_row)
