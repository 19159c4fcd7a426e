"""The oracle's decode step run over the sequences of a batch by several processes.

TEST INFRASTRUCTURE ONLY (the CPU-baseline leg of the benchmark and its test): the
arithmetic is sv_oracle's, unchanged and called as it stands; this module only
splits the batch by sequence, hands each slice to a worker process and puts the
results back together.  Everything except the length selection is independent per
sequence (Sec. 5 of the SV paper couples the sequences of a batch only through the
batch-greedy selection), so the step runs in two parallel phases around the
selection, which the parent process does itself:

    phase 1 (per slice)  row_stats, accept_estimate
    parent               select_length on the whole batch
    phase 2 (per slice)  verify_sample, with the Philox uniforms of the slice's
                         own sequence indices

Workers are started with the `spawn` method (fresh interpreters that import only
NumPy and this package) and read the logits from `.npy` files memory-mapped from a
directory the caller names (put it in /dev/shm), so nothing large is pickled.
"""
from __future__ import annotations

import multiprocessing as mp
import os

import numpy as np

from . import philox
from . import sv_oracle as O

_FILES = ("z_t", "z_d", "z_c", "x")


def save_inputs(directory, z_t, z_d, z_c, x):
    """Write the stored logits (float32, or bfloat16 as uint16 bit patterns) and the
    drafted tokens where the workers can map them."""
    os.makedirs(directory, exist_ok=True)
    for name, a in zip(_FILES, (z_t, z_d, z_c, x)):
        np.save(os.path.join(directory, name + ".npy"), np.ascontiguousarray(a))


def remove_inputs(directory):
    for name in _FILES:
        p = os.path.join(directory, name + ".npy")
        if os.path.exists(p):
            os.remove(p)
    if os.path.isdir(directory) and not os.listdir(directory):
        os.rmdir(directory)


def _load(directory, name):
    return np.load(os.path.join(directory, name + ".npy"), mmap_mode="r")


def _phase1(args):
    directory, lo, hi, edges_s, edges_a, table = args
    z_d, z_c, x = (_load(directory, n) for n in ("z_d", "z_c", "x"))
    r = O.row_stats(z_d[lo:hi], z_c[lo:hi], x[lo:hi])
    p_hat, _ = O.accept_estimate(r["S"].astype(np.float32), r["A"].astype(np.float32), edges_s, edges_a, table)
    return lo, hi, r["S"], r["A"], p_hat


def _phase2(args):
    directory, lo, hi, gamma, t_offsets, seed, step, cdf_abs_band = args
    z_t, z_d, x = (_load(directory, n) for n in ("z_t", "z_d", "x"))
    k = z_d.shape[1]
    seq = np.arange(lo, hi)[:, None]
    # the oracle addresses its uniforms by the position of a sequence in what it is given:
    # hand it those of the slice's own sequence indices
    ua, _ = philox.sv_uniforms(seed, step, np.broadcast_to(seq, (hi - lo, k)), np.arange(k)[None, :])
    _, us = philox.sv_uniforms(seed, step, np.broadcast_to(seq, (hi - lo, k + 1)), np.arange(k + 1)[None, :])
    g = None if gamma is None else gamma[lo:hi]
    if t_offsets is None:
        ref = O.verify_sample(z_t[lo:hi], z_d[lo:hi], x[lo:hi], gamma=g, uniforms=(ua, us),
                              cdf_abs_band=cdf_abs_band)
    else:
        ref = O.verify_sample(z_t, z_d[lo:hi], x[lo:hi], gamma=g, t_offsets=t_offsets[lo:hi + 1],
                              uniforms=(ua, us), cdf_abs_band=cdf_abs_band)
    return lo, hi, {n: ref[n] for n in ("tokens", "n_accept", "flags")}


def slices(B, n):
    """B sequences in at most n contiguous slices of nearly equal size."""
    n = max(1, min(n, B))
    cuts = [(B * j) // n for j in range(n + 1)]
    return [(cuts[j], cuts[j + 1]) for j in range(n) if cuts[j + 1] > cuts[j]]


def make_pool(n_workers):
    """A pool of n_workers fresh interpreters, started and warmed up (so that no timing
    that follows includes their start)."""
    pool = mp.get_context("spawn").Pool(n_workers)
    pool.map(abs, range(n_workers))
    return pool


def step(pool, n_workers, directory, B, edges_s, edges_a, table, latency, seed=0, step_index=0,
         verify_selected=False, packed=False, cdf_abs_band=0.0):
    """One whole decode step of the oracle on the batch saved under `directory`.

    verify_selected: verify the lengths the selection chose (else all k drafted tokens);
    packed: z_t.npy holds the packed target rows [sum_b (gamma_b + 1), V] of exactly those
    lengths.  Returns dict(S, A, p_hat, gamma, t_offsets, total_M, tokens, n_accept, flags).
    """
    sl = slices(B, n_workers)
    S = A = p_hat = None
    for lo, hi, s_, a_, p_ in pool.map(_phase1, [(directory, lo, hi, edges_s, edges_a, table) for lo, hi in sl]):
        if S is None:
            k = s_.shape[1]
            S, A = np.empty((B, k)), np.empty((B, k))
            p_hat = np.empty((B, k), dtype=np.float32)
        S[lo:hi], A[lo:hi], p_hat[lo:hi] = s_, a_, p_
    gamma, t_offsets, total = O.select_length(p_hat, latency)
    g = gamma if verify_selected else None
    offs = t_offsets if packed else None
    out = dict(S=S, A=A, p_hat=p_hat, gamma=gamma, t_offsets=t_offsets, total_M=total)
    parts = pool.map(_phase2, [(directory, lo, hi, g, offs, seed, step_index, cdf_abs_band) for lo, hi in sl])
    k1 = parts[0][2]["tokens"].shape[1]
    out["tokens"] = np.empty((B, k1), dtype=np.int32)
    out["n_accept"] = np.empty(B, dtype=np.int32)
    out["flags"] = np.empty(B, dtype=np.uint32)
    for lo, hi, r in parts:
        for n in ("tokens", "n_accept", "flags"):
            out[n][lo:hi] = r[n]
    return out
