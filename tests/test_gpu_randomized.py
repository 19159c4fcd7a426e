"""Randomised GPU parity sweep: many small seeded problems with mixed shapes,
dtypes, noise scales, verification lengths and Philox seeds, so that rare
near-tie / CDF-edge situations and odd shapes get exercised."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(6))
def test_random_problems(block):
    rng = np.random.default_rng(9000 + block)
    n_tie = n_edge = n_seq = 0
    for case in range(10):
        idx = int(rng.integers(0, 4))
        B = int(rng.integers(1, 9))
        k = int(rng.integers(1, 10))
        V = int(rng.choice([int(rng.integers(2, 300)), int(rng.integers(300, 9000)),
                            8 * int(rng.integers(1000, 5000)), 8192 * int(rng.integers(1, 4)) + int(rng.integers(0, 9))]))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        seed = int(rng.integers(0, 2 ** 31))
        cfg = svgen.make_config(idx, B=B, k=k, V=V, dtype=dtype, seed=seed)
        d = {n: cfg[n].cuda() for n in ("z_t", "z_d", "z_c", "x")}
        oi = H.oracle_inputs(cfg)
        ref = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
        with_kl = bool(rng.random() < 0.5)
        H.assert_row_stats(H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl), ref, with_kl)
        gamma = rng.integers(0, k + 1, size=B).astype(np.int32) if rng.random() < 0.6 else None
        pseed, step = int(rng.integers(0, 2 ** 62)), int(rng.integers(0, 2 ** 31))
        vref = O.verify_sample(oi["z_t"], oi["z_d"], oi["x"], gamma=gamma, seed=pseed, step=step)
        vgot = H.gpu_verify(d["z_t"], d["z_d"], d["x"], gamma=gamma, seed=pseed, step=step)
        t, e = H.assert_verify(vgot, vref, k)
        n_tie, n_edge, n_seq = n_tie + t, n_edge + e, n_seq + B
        p = rng.random((B, k)).astype(np.float32)
        lat = svgen.latency_table(B * k, t0=float(rng.uniform(0.1, 30)), d=float(rng.uniform(0.01, 1)),
                                  m0=int(rng.integers(1, B * k + 1)))
        for mode, l in ((O.MODE_BATCH_GREEDY, lat), (O.MODE_PER_SEQUENCE, lat[:k + 1])):
            rg, ro, rm = O.select_length(p, l, mode)
            gg, go, gm = H.gpu_select_length(p, l, mode)
            assert gm == rm and np.array_equal(gg, rg) and np.array_equal(go, ro)
    print(f"\n  block {block}: {n_seq} sequences, near-tie {n_tie}, near-cdf-edge {n_edge}", flush=True)
