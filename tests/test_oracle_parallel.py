"""The multi-process run of the oracle (the N-core CPU baseline of the benchmark) must give
exactly what the single-process oracle gives: it is the same arithmetic on slices."""
import os
import tempfile

import numpy as np

import svgen
from oracle import parallel as OP
from oracle import sv_oracle as O


def test_parallel_step_equals_single_process():
    B, k, V = 5, 3, 700
    cfg = svgen.make_config(1, B=B, k=k, V=V, dtype="bf16", seed=99)
    zt, zd, zc = (svgen.to_numpy_bits(cfg[n]) for n in ("z_t", "z_d", "z_c"))
    x = cfg["x"].numpy()
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = svgen.latency_table(B * k)
    r = O.row_stats(zd, zc, x)
    p, _ = O.accept_estimate(r["S"].astype(np.float32), r["A"].astype(np.float32), edges_s, edges_a, table)
    g, offs, total = O.select_length(p, lat)
    base = "/dev/shm" if os.path.isdir("/dev/shm") else None
    d = tempfile.mkdtemp(prefix="svpar_", dir=base)
    pool = OP.make_pool(2)
    try:
        OP.save_inputs(d, zt, zd, zc, x)
        full = OP.step(pool, 2, d, B, edges_s, edges_a, table, lat, seed=3, step_index=4)
        ref = O.verify_sample(zt, zd, x, seed=3, step=4)
        assert np.array_equal(full["S"], r["S"]) and np.array_equal(full["A"], r["A"])
        assert np.array_equal(full["p_hat"], p) and np.array_equal(full["gamma"], g)
        assert np.array_equal(full["t_offsets"], offs) and full["total_M"] == total
        for n in ("tokens", "n_accept", "flags"):
            assert np.array_equal(full[n], ref[n]), n
        # the ragged chain: packed target rows of the selected lengths
        packed = np.concatenate([zt[b, :g[b] + 1] for b in range(B)], axis=0)
        OP.save_inputs(d, packed, zd, zc, x)
        rag = OP.step(pool, 2, d, B, edges_s, edges_a, table, lat, seed=3, step_index=4,
                      verify_selected=True, packed=True)
        ref = O.verify_sample(packed, zd, x, gamma=g, t_offsets=offs, seed=3, step=4)
        for n in ("tokens", "n_accept", "flags"):
            assert np.array_equal(rag[n], ref[n]), n
    finally:
        pool.close()
        pool.join()
        OP.remove_inputs(d)
    assert not os.path.exists(d)
    assert OP.slices(5, 8) == [(0, 1), (1, 2), (2, 3), (3, 4), (4, 5)] and OP.slices(7, 2) == [(0, 3), (3, 7)]
