"""GPU parity: every C-ABI call against the CPU oracle on the same seeded
inputs, element by element.  Stage-isolated: each call is fed the oracle's
upstream outputs so that an upstream near-edge difference cannot hide or fake
a downstream one; the chained step is checked separately."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu

# (config recipe, B, k, V, dtype): small enough for the oracle to finish in
# seconds, spanning several vector tiles, ragged tails and unaligned rows.
SMALL = [
    (0, 1, 4, 32000, "f32"),      # config 1 at full size
    (1, 8, 8, 32000, "bf16"),     # config 2 at full size
    (0, 2, 3, 4099, "f32"),       # odd V: rows not 16-byte aligned -> scalar path
    (1, 3, 2, 8200 + 3, "bf16"),  # odd V bf16
    (3, 4, 3, 8192 * 2 + 8, "bf16"),   # just over two sampling chunks
    (2, 3, 2, 20000, "bf16"),     # heavy-tailed rows
    (1, 2, 5, 7, "bf16"),         # tiny vocabulary
    (0, 2, 2, 1, "f32"),          # single-entry vocabulary
    (1, 2, 3, 8, "bf16"),         # one 16-byte vector per row (aligned path, everything in registers)
    (0, 3, 2, 4, "f32"),          # the same for fp32
    (3, 2, 2, 5128, "bf16"),      # aligned rows shorter than the register share of the parking kernel
    (3, 1, 2, 131072 + 64, "bf16"),  # reaches past the register and LDS shares into the re-read region
]


def _gen(idx, B, k, V, dtype):
    cfg = svgen.make_config(idx, B=B, k=k, V=V, dtype=dtype)
    dev = {n: cfg[n].cuda() for n in ("z_t", "z_d", "z_c", "x")}
    return cfg, dev


@pytest.mark.parametrize("idx,B,k,V,dtype", SMALL)
@pytest.mark.parametrize("with_kl", [True, False])
def test_row_stats(idx, B, k, V, dtype, with_kl):
    cfg, d = _gen(idx, B, k, V, dtype)
    oi = H.oracle_inputs(cfg)
    ref = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
    got = H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl)
    H.assert_row_stats(got, ref, with_kl)


@pytest.mark.parametrize("idx,B,k,V,dtype", SMALL)
def test_verify_sample_dense(idx, B, k, V, dtype):
    cfg, d = _gen(idx, B, k, V, dtype)
    oi = H.oracle_inputs(cfg)
    for seed, step in ((0, 0), (0xDEADBEEF12345, 7)):
        ref = H.oracle_verify(oi["z_t"], oi["z_d"], oi["x"], seed=seed, step=step)
        got = H.gpu_verify(d["z_t"], d["z_d"], d["x"], seed=seed, step=step)
        H.assert_verify(got, ref, k)


@pytest.mark.parametrize("idx,B,k,V,dtype", SMALL[:6])
def test_verify_sample_gamma_and_packed(idx, B, k, V, dtype):
    cfg, d = _gen(idx, B, k, V, dtype)
    oi = H.oracle_inputs(cfg)
    rng = np.random.default_rng(idx + B)
    gamma = rng.integers(0, k + 1, size=B).astype(np.int32)
    gamma[0] = 0
    ref = H.oracle_verify(oi["z_t"], oi["z_d"], oi["x"], gamma=gamma, seed=3, step=1)
    got = H.gpu_verify(d["z_t"], d["z_d"], d["x"], gamma=gamma, seed=3, step=1)
    H.assert_verify(got, ref, k)
    offs = np.concatenate([[0], np.cumsum(gamma + 1)]).astype(np.int32)
    packed = torch.cat([d["z_t"][b, :gamma[b] + 1] for b in range(B)]).contiguous()
    got = H.gpu_verify(packed, d["z_d"], d["x"], gamma=gamma, t_offsets=offs, seed=3, step=1)
    H.assert_verify(got, ref, k)


def test_accept_estimate_exact():
    rng = np.random.default_rng(0)
    for n_s, n_a in ((5, 5), (10, 10), (20, 20), (16, 17), (1, 1)):
        edges_s = np.sort(np.concatenate([[0, 1], rng.random(n_s - 1)])).astype(np.float32)
        edges_a = np.linspace(0, 1, n_a + 1).astype(np.float32)
        table = rng.random((n_s, n_a)).astype(np.float32)
        S = rng.random(3000).astype(np.float32)
        A = np.minimum(1, 1.3 * rng.random(3000)).astype(np.float32)
        S[:n_s + 1] = edges_s
        A[:n_a + 1] = edges_a
        S[40:44] = [np.nan, -1.0, 2.0, 1.0]
        A[44:46] = [np.nan, 1.0]
        S[50:60] = edges_s[min(1, n_s)] + np.float32(1e-5) * np.linspace(-2, 2, 10, dtype=np.float32)
        ref_p, ref_f = O.accept_estimate(S, A, edges_s, edges_a, table)
        got_p, got_f = H.gpu_accept_estimate(S, A, edges_s, edges_a, table)
        assert np.array_equal(got_p, ref_p)
        assert np.array_equal(got_f, ref_f)


@pytest.mark.parametrize("B,k", [(1, 4), (8, 8), (64, 8), (64, 16), (3, 5), (4096, 1), (1, 64), (37, 11), (512, 16), (300, 20),
                                 (8192, 1)])
def test_select_length_exact(B, k):
    rng = np.random.default_rng(B * 100 + k)
    for trial in range(3):
        p = rng.random((B, k)).astype(np.float32)
        if trial == 1:
            p = np.round(p * 4) / 4            # many ties, zeros and ones
            p = p.astype(np.float32)
        if trial == 2:
            p[rng.random((B, k)) < 0.05] = np.nan
            p[0, 0] = 1.5
        lat_b = svgen.latency_table(B * k, t0=float(rng.uniform(0.1, 30)), d=0.08, m0=max(1, B * k // 4))
        for mode, lat in ((O.MODE_BATCH_GREEDY, lat_b), (O.MODE_PER_SEQUENCE, lat_b[:k + 1])):
            rg, ro, rm = O.select_length(p, lat, mode)
            gg, go, gm = H.gpu_select_length(p, lat, mode)
            assert gm == rm
            assert np.array_equal(gg, rg)
            assert np.array_equal(go, ro)


def test_select_length_degenerate():
    for p in (np.zeros((5, 4), np.float32), np.ones((5, 4), np.float32)):
        for lat in (np.ones(21, np.float32), (10.0 ** np.arange(21)).astype(np.float32)):
            rg, ro, rm = O.select_length(p, lat)
            gg, go, gm = H.gpu_select_length(p, lat, 0)
            assert gm == rm and np.array_equal(gg, rg) and np.array_equal(go, ro)


def test_chained_step_config2():
    """The four calls chained on device buffers (no host round trip), against
    the oracle chained the same way."""
    import paper_2509_24328_amd as P
    cfg, d = _gen(1, 8, 8, 32000, "bf16")
    oi = H.oracle_inputs(cfg)
    B, k, V = 8, 8, 32000
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = svgen.latency_table(B * k)
    f = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    lse_d, lse_c, S, A, p_hat = f(B, k), f(B, k), f(B, k), f(B, k), f(B, k)
    eflag = torch.empty((B, k), dtype=torch.uint8, device="cuda")
    gamma = torch.empty(B, dtype=torch.int32, device="cuda")
    offs = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    total = torch.empty(1, dtype=torch.int32, device="cuda")
    tokens = torch.empty((B, k + 1), dtype=torch.int32, device="cuda")
    n_acc = torch.empty(B, dtype=torch.int32, device="cuda")
    flags = torch.empty(B, dtype=torch.int32, device="cuda")
    ratio = f(B, k)
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    P.sv_row_stats(d["z_d"], d["z_c"], d["x"], lse_d, lse_c, S, A, None, None, ws)
    P.sv_accept_estimate(S, A, H.dev(edges_s), H.dev(edges_a), H.dev(table), p_hat, eflag)
    P.sv_select_length(p_hat, H.dev(lat), P.SV_BATCH_GREEDY, gamma, offs, total)
    P.sv_verify_sample(d["z_t"], None, d["z_d"], d["x"], gamma, 0, 0, tokens, n_acc, flags, ratio, ws)
    torch.cuda.synchronize()

    r = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
    rp, rflag = O.accept_estimate(r["S"].astype(np.float32), r["A"].astype(np.float32),
                                  edges_s, edges_a, table)
    assert not rflag.any(), "seeded inputs sit on a bin edge; pick another seed"
    assert np.array_equal(p_hat.cpu().numpy(), rp)
    rg, ro, rm = O.select_length(rp, lat)
    assert np.array_equal(gamma.cpu().numpy(), rg) and int(total.item()) == rm
    assert np.array_equal(offs.cpu().numpy(), ro)
    ref = H.oracle_verify(oi["z_t"], oi["z_d"], oi["x"], gamma=rg)
    got = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
               flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
    H.assert_verify(got, ref, k)


def test_philox_uniforms_agree_on_a_million_counters():
    """The two independently written Philox generators (oracle/philox.py and the
    device one) on 2 * 10^6 uniforms: bit-identical doubles."""
    from oracle import philox as OP
    P = H.sv()
    B, n_pos = 1000, 1000
    for seed, step in ((0, 0), (0x0123456789ABCDEF, 7), ((1 << 64) - 1, (1 << 32) - 1)):
        ua = torch.empty((B, n_pos), dtype=torch.float64, device="cuda")
        us = torch.empty((B, n_pos), dtype=torch.float64, device="cuda")
        P.sv_uniforms(seed, step, ua, us)
        torch.cuda.synchronize()
        b = np.arange(B)[:, None]
        i = np.arange(n_pos)[None, :]
        ra, rs = OP.sv_uniforms(seed, step, b, i)
        assert np.array_equal(ua.cpu().numpy(), ra) and np.array_equal(us.cpu().numpy(), rs)


def test_select_length_many_ties_at_large_key_counts():
    """Thousands of keys with only a few distinct estimates: the tie order (lowest
    sequence first, then position) and the exact-sum fallback at every size class of
    the kernel (one key per lane, runs of keys, in-place merge)."""
    rng = np.random.default_rng(77)
    for B, k in ((100, 8), (250, 12), (400, 16), (512, 16)):
        p = rng.choice(np.array([1.0, 0.5, 0.25, 0.75], dtype=np.float32), size=(B, k))
        for lat in (svgen.latency_table(B * k), svgen.latency_table(B * k, t0=1.0, d=0.5, m0=4)):
            rg, ro, rm = O.select_length(p, lat, O.MODE_BATCH_GREEDY)
            gg, go, gm = H.gpu_select_length(p, lat, O.MODE_BATCH_GREEDY)
            assert gm == rm and np.array_equal(gg, rg) and np.array_equal(go, ro), (B, k)
