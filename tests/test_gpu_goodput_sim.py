"""The step-level goodput simulation through the C ABI against its oracle twin
(oracle/goodput_oracle.py): for plain SD and for the three acceptance estimators
((S, A), draft entropy, draft-token probability) the selected lengths, the number
of verified tokens and the accept counts of every step are integers and must be
identical; the totals follow.  Plus the qualitative effect the paper reports."""
import numpy as np
import pytest
import torch

import svgen
from oracle import goodput_oracle as GO
from oracle import profile_oracle as PO
from oracle import sv_oracle as O
import harness as H

pytestmark = pytest.mark.gpu


def _np(c):
    return tuple(svgen.to_numpy_bits(c[n]) for n in ("z_t", "z_d", "z_c")) + (c["x"].cpu().numpy(),)


def test_every_step_matches_the_oracle_exactly():
    from paper_2509_24328_amd import goodput_sim as G
    B, k, V, steps = 12, 6, 8192, 5
    mk = lambda seed: svgen.make_config(3, seed=seed, B=B, k=k, V=V, device="cuda")
    latency = svgen.latency_table(B * k, t0=5.0, d=0.5, m0=16)
    # profiles: built by the oracle on a held-out batch and handed to both sides (the GPU's own
    # profile pass is compared with the oracle's in test_gpu_profile.py)
    held = mk(4000)
    zt, zd, zc, x = _np(held)
    sig = GO.signals(zd, zc, x)
    ratio, _ = PO.accept_probability_ratio(zt, zd, x)
    prof = {m: GO.build_profile(m, sig, ratio, V, cells=16, n_x=8) for m in GO.ESTIMATORS}
    dprof = {m: tuple(H.dev(a) for a in prof[m][:3]) for m in prof}
    batches = [mk(4100 + t) for t in range(steps)]
    res = G.simulate(lambda t: batches[t], latency, steps, dprof, keep_steps=True)
    per_step, compared, skipped = [], 0, 0
    for t in range(steps):
        out, osig = GO.step(*_np(batches[t]), prof, latency, seed=1234, step_index=t)
        per_step.append(out)
        got = res["steps"][t]
        for n in ("S", "A", "H_d", "pd_x"):
            assert H.close(got["signals"][n], osig[n].astype(np.float64), H.REL, 2e-6).all(), (t, n)
        for m in ("sd",) + GO.ESTIMATORS:
            g, r = got[m], out[m]
            if g["near_edge"] or r["near_edge"]:        # a signal within 1e-5 of a bin edge: the two
                skipped += 1                            # sides may look up neighbouring cells
                continue
            assert np.array_equal(g["gamma"], r["gamma"]), (t, m, g["gamma"], r["gamma"])
            assert g["M"] == r["M"], (t, m)
            tie = r["near_tie"] | ((g["flags"] & O.FLAG_NEAR_TIE) != 0)
            assert np.array_equal(g["n_accept"][~tie], r["n_accept"][~tie]), (t, m)
            compared += 1
    assert compared >= 3 * steps, (compared, skipped)
    # totals: the same bookkeeping on both sides wherever every step was compared
    tot = GO.totals(per_step)
    for m in ("sd",) + GO.ESTIMATORS:
        same = all(not (res["steps"][t][m]["near_edge"] or per_step[t][m]["near_edge"])
                   and not per_step[t][m]["near_tie"].any() and
                   not (res["steps"][t][m]["flags"] & O.FLAG_NEAR_TIE).any() for t in range(steps))
        if same:
            assert res[m]["accepted"] == tot[m]["accepted"] and res[m]["verified"] == tot[m]["verified"]
            assert abs(res[m]["latency"] - tot[m]["latency"]) < 1e-9 * tot[m]["latency"]
            assert abs(res[m]["goodput"] - tot[m]["goodput"]) < 1e-9 * max(tot[m]["goodput"], 1e-30)
    print(f"\n  steps x estimators compared exactly {compared}, skipped for a bin-edge band {skipped}; "
          + ", ".join(f"{m}: goodput {res[m]['goodput']:.4f}" for m in ("sd",) + GO.ESTIMATORS), flush=True)


def test_sv_verifies_less_and_accepts_a_larger_fraction():
    from paper_2509_24328_amd import goodput_sim as G
    mk = lambda seed: svgen.make_config(3, seed=seed, B=16, k=8, V=16384, device="cuda")
    held = mk(777)
    latency = svgen.latency_table(16 * 8, t0=5.0, d=0.5, m0=16)
    profiles = G.build_profiles(held, cells=16, n_x=8)
    gain = {m: profiles[m][3][2] for m in profiles}
    assert gain["sv"] > 0                         # positive information gain on the held-out batch
    assert gain["sv"] > gain["entropy"] and gain["sv"] > gain["probability"], gain
    res = G.simulate(lambda t: mk(900 + t), latency, steps=6, profiles=profiles)
    sd, sv = res["sd"], res["sv"]
    print("\n  information gain (bits): " + ", ".join(f"{m} {gain[m]:.3f}" for m in gain))
    for m in ("sd",) + G.ESTIMATORS:
        r = res[m]
        print(f"  {m:12s} accept rate {r['accept_rate']:.3f}, verified/seq {r['mean_verified_per_seq']:.2f}, "
              f"goodput {r['goodput']:.4f}")
    assert sv["verified"] < sd["verified"]
    assert sv["accept_rate"] > sd["accept_rate"]
    assert sv["goodput"] > sd["goodput"]          # with a latency table that charges per verified token
    assert sv["goodput"] >= max(res["entropy"]["goodput"], res["probability"]["goodput"]) * 0.98


def test_warped_simulation_on_compacted_supports():
    """Same with the paper's sampling hyper-parameters in force (temperature 0.7,
    top-k 20, top-p 0.8), everything on compacted supports."""
    from paper_2509_24328_amd import goodput_sim as G
    warp = (float(np.float32(0.7)), 20, 0.8)
    mk = lambda seed: svgen.make_config(3, seed=seed, B=16, k=8, V=16384, device="cuda")
    held = mk(778)
    latency = svgen.latency_table(16 * 8, t0=5.0, d=0.5, m0=16)
    profile = G.build_profile(held, warp=warp)
    res = G.simulate(lambda t: mk(950 + t), latency, steps=6, profiles=profile, warp=warp)
    sd, sv = res["sd"], res["sv"]
    print(f"\n  warped SD: accept rate {sd['accept_rate']:.3f}, verified/seq {sd['mean_verified_per_seq']:.2f}, "
          f"goodput {sd['goodput']:.4f};  SV: accept rate {sv['accept_rate']:.3f}, "
          f"verified/seq {sv['mean_verified_per_seq']:.2f}, goodput {sv['goodput']:.4f}")
    assert sv["verified"] < sd["verified"]
    assert sv["accept_rate"] >= sd["accept_rate"]
