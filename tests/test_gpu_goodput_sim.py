"""The step-level goodput simulation runs end to end through the C ABI and
shows the qualitative effect the paper reports: choosing verification lengths
from the (S, A) estimate raises the fraction of verified tokens that are
accepted, at far fewer verified tokens."""
import pytest

import svgen

pytestmark = pytest.mark.gpu


def test_sv_verifies_less_and_accepts_a_larger_fraction():
    from paper_2509_24328_amd import goodput_sim as G
    mk = lambda seed: svgen.make_config(3, seed=seed, B=16, k=8, V=16384, device="cuda")
    held = mk(777)
    latency = svgen.latency_table(16 * 8, t0=5.0, d=0.5, m0=16)
    profile = G.build_profile(held)
    assert profile[3][2] > 0                      # positive information gain on the held-out batch
    res = G.simulate(lambda t: mk(900 + t), latency, steps=6, profile=profile)
    sd, sv = res["sd"], res["sv"]
    print(f"\n  SD: accept rate {sd['accept_rate']:.3f}, verified/seq {sd['mean_verified_per_seq']:.2f}, "
          f"goodput {sd['goodput']:.4f};  SV: accept rate {sv['accept_rate']:.3f}, "
          f"verified/seq {sv['mean_verified_per_seq']:.2f}, goodput {sv['goodput']:.4f}")
    assert sv["verified"] < sd["verified"]
    assert sv["accept_rate"] > sd["accept_rate"]
    assert sv["goodput"] > sd["goodput"]          # with a latency table that charges per verified token


def test_warped_simulation_on_compacted_supports():
    """Same with the paper's sampling hyper-parameters in force (temperature 0.7,
    top-k 20, top-p 0.8), everything on compacted supports."""
    import numpy as np
    from paper_2509_24328_amd import goodput_sim as G
    warp = (float(np.float32(0.7)), 20, 0.8)
    mk = lambda seed: svgen.make_config(3, seed=seed, B=16, k=8, V=16384, device="cuda")
    held = mk(778)
    latency = svgen.latency_table(16 * 8, t0=5.0, d=0.5, m0=16)
    profile = G.build_profile(held, warp=warp)
    res = G.simulate(lambda t: mk(950 + t), latency, steps=6, profile=profile, warp=warp)
    sd, sv = res["sd"], res["sv"]
    print(f"\n  warped SD: accept rate {sd['accept_rate']:.3f}, verified/seq {sd['mean_verified_per_seq']:.2f}, "
          f"goodput {sd['goodput']:.4f};  SV: accept rate {sv['accept_rate']:.3f}, "
          f"verified/seq {sv['mean_verified_per_seq']:.2f}, goodput {sv['goodput']:.4f}")
    assert sv["verified"] < sd["verified"]
    assert sv["accept_rate"] >= sd["accept_rate"]
