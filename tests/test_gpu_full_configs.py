"""GPU parity at the full sizes of the five workload configurations, in the
launch configuration bench.py times, on every output (the oracle finishes each
config in well under a minute).  Config 5 runs the whole chain with the ragged
layout: lengths from sv_select_length, target rows packed for the selected
positions plus the bonus row, int32 offsets."""
import time

import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu


def _stage_isolated(index):
    t0 = time.time()
    cfg = svgen.make_config(index)
    d = {n: cfg[n].cuda() for n in ("z_t", "z_d", "z_c", "x")}
    oi = H.oracle_inputs(cfg)
    B, k = cfg["B"], cfg["k"]
    print(f"\n[{cfg['name']}] generated in {time.time() - t0:.1f}s", flush=True)

    t0 = time.time()
    ref = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
    got = H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl=True)
    H.assert_row_stats(got, ref, True)
    got = H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl=False)
    H.assert_row_stats(got, ref, False)
    print(f"  row_stats ok ({time.time() - t0:.1f}s)", flush=True)

    edges_s, edges_a, table = svgen.profile_table(10, 10)
    S32, A32 = ref["S"].astype(np.float32), ref["A"].astype(np.float32)
    rp, rflag = O.accept_estimate(S32, A32, edges_s, edges_a, table)
    gp, gflag = H.gpu_accept_estimate(S32, A32, edges_s, edges_a, table)
    assert np.array_equal(gp, rp) and np.array_equal(gflag, rflag)

    lat = svgen.latency_table(B * k)
    for mode, l in ((O.MODE_BATCH_GREEDY, lat), (O.MODE_PER_SEQUENCE, lat[:k + 1])):
        rg, ro, rm = O.select_length(rp, l, mode)
        gg, go, gm = H.gpu_select_length(rp, l, mode)
        assert gm == rm and np.array_equal(gg, rg) and np.array_equal(go, ro)
    print("  accept_estimate / select_length ok", flush=True)
    return cfg, d, oi, rp, lat


@pytest.mark.parametrize("index", [2, 3])
def test_full_config_dense(index):
    cfg, d, oi, rp, lat = _stage_isolated(index)
    k = cfg["k"]
    t0 = time.time()
    ref = O.verify_sample(oi["z_t"], oi["z_d"], oi["x"], seed=0, step=0)
    got = H.gpu_verify(d["z_t"], d["z_d"], d["x"], seed=0, step=0)
    n_tie, n_edge = H.assert_verify(got, ref, k)
    print(f"  verify (gamma = k) ok: near-tie {n_tie}, near-cdf-edge {n_edge}, "
          f"mean accepted {ref['n_accept'].mean():.2f} ({time.time() - t0:.1f}s)", flush=True)
    rg, _, _ = O.select_length(rp, lat)
    ref = O.verify_sample(oi["z_t"], oi["z_d"], oi["x"], gamma=rg, seed=1, step=3)
    got = H.gpu_verify(d["z_t"], d["z_d"], d["x"], gamma=rg, seed=1, step=3)
    n_tie, n_edge = H.assert_verify(got, ref, k)
    print(f"  verify (selected gamma, mean {rg.mean():.2f}) ok: near-tie {n_tie}, near-cdf-edge {n_edge}",
          flush=True)


def test_full_config5_ragged_chain():
    cfg, d, oi, rp, lat = _stage_isolated(4)
    B, k = cfg["B"], cfg["k"]
    rg, ro, rm = O.select_length(rp, lat)
    assert 0 < rm < B * k, "the latency table should make the selection non-trivial"
    # the caller packs the target rows of the selected positions + bonus row
    packed = torch.cat([d["z_t"][b, :rg[b] + 1] for b in range(B)]).contiguous()
    packed_np = np.concatenate([oi["z_t"][b, :rg[b] + 1] for b in range(B)])
    assert packed.shape[0] == ro[-1]
    ref = O.verify_sample(packed_np, oi["z_d"], oi["x"], gamma=rg, t_offsets=ro, seed=5, step=2)
    got = H.gpu_verify(packed, d["z_d"], d["x"], gamma=rg, t_offsets=ro, seed=5, step=2)
    n_tie, n_edge = H.assert_verify(got, ref, k)
    full = int((ref["n_accept"] == rg).sum())
    early = int(((ref["n_accept"] < rg) & (rg > 0)).sum())
    print(f"  ragged verify ok: sum gamma {rm}, packed rows {ro[-1]}, full-accept rows {full}, "
          f"early-stop rows {early}, gamma=0 rows {int((rg == 0).sum())}, near-tie {n_tie}, "
          f"near-cdf-edge {n_edge}", flush=True)
    # dense layout with the same lengths must agree with the packed one
    got_dense = H.gpu_verify(d["z_t"], d["z_d"], d["x"], gamma=rg, seed=5, step=2)
    assert np.array_equal(got_dense["tokens"], got["tokens"])
    assert np.array_equal(got_dense["n_accept"], got["n_accept"])
