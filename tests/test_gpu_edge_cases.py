"""GPU parity on the degenerate inputs of the method: bad rows, impossible
tokens, zero verification length, identical models, masked vocabularies."""
import numpy as np
import pytest
import torch

from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu


def _case(B=4, k=3, V=300, seed=0, dtype=torch.float32):
    rng = np.random.default_rng(seed)
    z_t = (2 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    z_d = (z_t[:, :k] + rng.standard_normal((B, k, V))).astype(np.float32)
    z_c = (z_t[:, :k] + rng.standard_normal((B, k, V))).astype(np.float32)
    x = rng.integers(0, V, size=(B, k)).astype(np.int32)
    return z_t, z_d, z_c, x


def _run_verify(z_t, z_d, x, **kw):
    ref = H.oracle_verify(z_t, z_d, x, **kw)
    got = H.gpu_verify(H.dev(z_t), H.dev(z_d), H.dev(x), **kw)
    return got, ref


def test_empty_batch_is_a_no_op():
    import paper_2509_24328_amd as P
    e = torch.empty(0, device="cuda")
    ws = P.alloc_workspace(0, 4, 100, P.SV_F32)
    assert P.binding.lib.sv_row_stats(None, None, None, 0, 4, 100, P.SV_F32, None, None, None, None,
                                      None, None, None, None, None, 0, None) == 0
    assert P.binding.lib.sv_verify_sample(None, None, 0, None, None, None, 0, 4, 100, P.SV_F32, 0, 0,
                                          None, None, None, None, None, 0, None) == 0
    assert P.binding.lib.sv_accept_estimate(None, None, 0, None, 3, None, 3, None, None, None, None) == 0
    torch.cuda.synchronize()
    del e, ws


def test_bad_rows_and_tokens_in_row_stats():
    z_t, z_d, z_c, x = _case()
    z_d[0, 0, 5] = np.nan
    z_c[1, 1, :] = -np.inf
    z_d[2, 2, 7] = np.inf
    x[3, 0] = -1
    x[3, 1] = 300
    z_d[3, 2, x[3, 2]] = -np.inf          # drafted token the draft could not have produced
    z_c[0, 1, 10:200] = -np.inf           # masked vocabulary entries are fine
    ref = O.row_stats(z_d, z_c, x)
    got = H.gpu_row_stats(H.dev(z_d), H.dev(z_c), H.dev(x))
    H.assert_row_stats(got, ref)
    assert got["A"][3, 2] == 1.0 and np.isinf(got["KL"][0, 1])


def test_bad_rows_and_tokens_in_verify():
    z_t, z_d, z_c, x = _case(B=6)
    z_t[0, 0, 3] = np.nan                 # first target row bad: nothing can be drawn
    z_d[1, 1, 3] = np.nan                 # draft row bad at position 1
    x[2, 0] = 999                         # token out of range
    z_t[3, 2, :] = -np.inf                # all -inf target row
    z_d[4, 0, x[4, 0]] = -np.inf          # p_d(x) = 0 -> ratio inf -> accepted
    z_t[5, 0, x[5, 0]] = -np.inf          # p_t(x) = 0 -> ratio 0 -> rejected
    for seed in range(4):
        got, ref = _run_verify(z_t, z_d, x, seed=seed)
        H.assert_verify(got, ref, 3)
        assert got["tokens"][0, 0] == -1 and got["flags"][0] & O.FLAG_BAD_ROW
        assert got["flags"][2] & O.FLAG_BAD_TOKEN and got["n_accept"][2] == 0
        assert got["n_accept"][5] == 0 and got["n_accept"][4] >= 1


def test_identical_models_accept_all_and_zero_gamma():
    z_t, _, _, x = _case(B=5, k=4, V=1000, seed=2)
    z_d = z_t[:, :4].copy()
    got, ref = _run_verify(z_t, z_d, x, seed=9)
    H.assert_verify(got, ref, 4)
    assert np.all(got["n_accept"] == 4)
    gamma = np.zeros(5, np.int32)
    got, ref = _run_verify(z_t, z_d, x, gamma=gamma, seed=9)
    H.assert_verify(got, ref, 4)
    assert np.all(got["n_accept"] == 0) and np.all(got["tokens"][:, 0] >= 0)


def test_disjoint_supports_and_one_hot_target():
    B, k, V = 3, 2, 64
    z_t = np.full((B, k + 1, V), -np.inf, np.float32)
    z_d = np.full((B, k, V), -np.inf, np.float32)
    z_t[:, :, :32] = 0.0
    z_d[:, :, 32:] = 0.0
    z_t[2, 0, :] = -np.inf
    z_t[2, 0, 17] = 2.0                   # one-hot target row
    x = np.full((B, k), 40, np.int32)
    for seed in range(3):
        got, ref = _run_verify(z_t, z_d, x, seed=seed)
        H.assert_verify(got, ref, k)
        assert np.all(got["n_accept"] == 0) and np.all(got["tokens"][:, 0] < 32)
        assert got["tokens"][2, 0] == 17


def test_packed_offsets_out_of_range_are_flagged_not_read():
    z_t, z_d, z_c, x = _case(B=3, k=2, V=128)
    gamma = np.array([2, 1, 2], np.int32)
    offs = np.array([0, 3, 5, 8], np.int32)
    packed = np.concatenate([z_t[b, :gamma[b] + 1] for b in range(3)])
    short = packed[:6]                    # sequence 2 now points past the buffer
    got = H.gpu_verify(H.dev(short), H.dev(z_d), H.dev(x), gamma=gamma, t_offsets=offs, seed=1)
    ref = H.oracle_verify(packed, z_d, x, gamma=gamma, t_offsets=offs, seed=1)
    for b in range(2):
        assert np.array_equal(got["tokens"][b], ref["tokens"][b])
    assert got["flags"][2] & O.FLAG_BAD_ROW


def test_results_are_reproducible_run_to_run():
    z_t, z_d, z_c, x = _case(B=8, k=4, V=5000, seed=5)
    a = H.gpu_verify(H.dev(z_t), H.dev(z_d), H.dev(x), seed=4)
    s1 = H.gpu_row_stats(H.dev(z_d), H.dev(z_c), H.dev(x))
    for _ in range(3):
        b = H.gpu_verify(H.dev(z_t), H.dev(z_d), H.dev(x), seed=4)
        s2 = H.gpu_row_stats(H.dev(z_d), H.dev(z_c), H.dev(x))
        for n in ("tokens", "n_accept", "flags"):
            assert np.array_equal(a[n], b[n])
        assert np.array_equal(a["ratio"], b["ratio"], equal_nan=True)
        for n in ("lse_d", "S", "A", "KL"):
            assert np.array_equal(s1[n], s2[n], equal_nan=True)


def test_kernels_with_floating_point_atomics_reproduce_their_outputs():
    """Two kernels add floating-point numbers with atomics, in whatever order the hardware
    serves them: the radix fallback of the warp kernel (fp64 bin masses in LDS) and the
    profile histogram (fp64 per-cell sums of X in global memory).  What they hand on is
    discrete or rounded far above that noise - a cutoff is a value of the row, and a top-p
    decision within 3e-6 of P is flagged; counts are integers; the table is an fp32 mean -
    so those outputs repeat bit for bit; the fp64 sums themselves repeat to 1e-15."""
    P = H.sv()
    rng = np.random.default_rng(12)
    rows, V = 6, 40000
    flat = (rng.standard_normal((rows, V)) * 0.01).astype(np.float32)    # flat rows take the radix path
    z = H.dev(flat)
    runs = []
    for _ in range(4):
        cut = torch.empty(rows, dtype=torch.float32, device="cuda")
        fl = torch.zeros(rows, dtype=torch.int32, device="cuda")
        P.sv_warp_cutoffs(z, 1.0, 0, 0.9, cut, fl)
        torch.cuda.synchronize()
        runs.append((cut.cpu().numpy(), fl.cpu().numpy()))
    for c, f in runs[1:]:
        assert np.array_equal(c, runs[0][0]) and np.array_equal(f, runs[0][1])
    n, n_s, n_a, n_x = 6000, 7, 5, 9
    S, A = rng.random(n).astype(np.float32), rng.random(n).astype(np.float32)
    ratio = (rng.random(n) * 1.3).astype(np.float32)
    es, ea = H.dev(np.linspace(0, 1, n_s + 1).astype(np.float32)), H.dev(np.linspace(0, 1, n_a + 1).astype(np.float32))
    outs = []
    for _ in range(4):
        counts = torch.zeros((n_s, n_a, n_x), dtype=torch.int32, device="cuda")
        sum_x = torch.zeros((n_s, n_a), dtype=torch.float64, device="cuda")
        table = torch.empty((n_s, n_a), dtype=torch.float32, device="cuda")
        info = torch.zeros(3, dtype=torch.float64, device="cuda")
        P.sv_profile_accumulate(H.dev(S), H.dev(A), H.dev(ratio), es, ea, n_x, counts, sum_x)
        P.sv_profile_finalize(counts, sum_x, table, info)
        torch.cuda.synchronize()
        outs.append((counts.cpu().numpy(), sum_x.cpu().numpy(), table.cpu().numpy(), info.cpu().numpy()))
    for c, sx, t, i in outs[1:]:
        assert np.array_equal(c, outs[0][0]) and np.array_equal(t, outs[0][2])
        assert np.allclose(sx, outs[0][1], rtol=1e-15, atol=0) and np.allclose(i, outs[0][3], rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("V,dtype", [(70000, torch.bfloat16), (40000, torch.float32), (152064, torch.bfloat16)])
def test_row_stats_when_the_running_reference_has_to_move(V, dtype):
    """The online sum-exp of sv_row_stats rescales its per-lane sums whenever the running
    maximum moves.  Rows that force that at every stage of the aligned-row kernel (sizes
    whose pairs span its register, LDS and re-read shares): steep ramps (up: a move every
    vector; down: none, later terms underflow), a row whose first half is masked, a row of
    -1e30 with a few ordinary entries, isolated spikes, and bad entries met late."""
    rng = np.random.default_rng(V)
    B, k = 2, 4
    base = (2 * rng.standard_normal((B, k, V))).astype(np.float32)
    ramp = np.linspace(-300.0, 300.0, V, dtype=np.float32)
    z_d = base.copy()
    z_c = (base + rng.standard_normal((B, k, V))).astype(np.float32)
    z_d[0, 0] += ramp                      # rising: the reference keeps moving
    z_c[0, 0] += 0.5 * ramp
    z_d[0, 1] += ramp[::-1]                # falling: no move, later terms underflow
    z_c[0, 1] += 0.9 * ramp[::-1]
    z_d[0, 2, : V // 2] = -np.inf          # nothing finite for the first half of the row
    z_c[0, 3, :] = -1e30                   # a reference far below the few ordinary entries
    z_c[0, 3, V // 3 :: 997] = base[0, 3, V // 3 :: 997]
    z_d[1, 0, V - 5] = np.nan              # bad entries met after the references are set
    z_c[1, 1, V - 9] = np.inf
    z_d[1, 2, 17::4096] += 200.0           # isolated spikes
    z_c[1, 3, 5::8192] += 90.0
    x = rng.integers(V // 2, V, size=(B, k)).astype(np.int32)
    if dtype == torch.bfloat16:            # the oracle sees exactly the stored values
        z_d = torch.from_numpy(z_d).to(torch.bfloat16).float().numpy()
        z_c = torch.from_numpy(z_c).to(torch.bfloat16).float().numpy()
    ref = O.row_stats(z_d, z_c, x)
    got = H.gpu_row_stats(H.dev(z_d, dtype), H.dev(z_c, dtype), H.dev(x))
    H.assert_row_stats(got, ref)
    assert np.isnan(got["lse_d"][1, 0]) and np.isnan(got["lse_c"][1, 1])
    assert np.isfinite(got["S"][0]).all()


@pytest.mark.parametrize("V,dtype,mask", [(301, torch.float32, -1e30), (4096, torch.bfloat16, -1e30),
                                          (300, torch.float32, float(np.finfo(np.float32).min)),
                                          (4096, torch.bfloat16, -3.3895313892515355e38), (2048, torch.float32, -1e10)])
def test_finite_stand_ins_for_minus_inf(V, dtype, mask):
    """Vocabulary masks written as a huge negative finite number instead of -inf carry no
    mass in any call (the library documents this range rule; in fp64 the oracle gets the
    same numbers because exp(mask - lse) underflows to zero)."""
    z_t, z_d, z_c, x = _case(B=3, k=3, V=V, seed=V)
    rng = np.random.default_rng(V + 1)
    for z in (z_t, z_d, z_c):
        z[rng.random(z.shape) < 0.7] = mask
    z_d[0, 0, :64] = mask                  # whole leading vectors masked
    z_t[1, 1, : V // 2] = mask
    z_d[2, 2, :] = mask                    # nothing in range: a bad row on the GPU ...
    z_d[2, 2, 0] = 1.0                     # ... unless one entry is
    x[0, 0] = 100
    if dtype == torch.bfloat16:
        z_t, z_d, z_c = (torch.from_numpy(z).to(torch.bfloat16).float().numpy() for z in (z_t, z_d, z_c))
    with np.errstate(over="ignore"):       # exp(-mask) overflows to +inf inside the oracle's min(1, .)
        ref = O.row_stats(z_d, z_c, x)
    # (KL is left out: draft mass on a masked companion entry makes it about -mask)
    got = H.gpu_row_stats(H.dev(z_d, dtype), H.dev(z_c, dtype), H.dev(x), with_kl=False)
    H.assert_row_stats(got, ref, with_kl=False)
    gotv, refv = _run_verify(z_t, z_d, x, seed=11, step=2) if dtype == torch.float32 else (None, None)
    if gotv is not None:
        H.assert_verify(gotv, refv, 3)


def test_longest_draft_fully_accepted():
    """k = 64 is the longest draft the verification accepts; when all 64 tokens are accepted
    the sampled position is the bonus row, number 64."""
    B, k, V = 3, 64, 500
    z_t, z_d, z_c, x = _case(B=B, k=k, V=V, seed=64)
    z_d[0] = z_t[0, :k]                    # identical models: every ratio is 1
    z_d[2] = z_t[2, :k]
    x[0] = np.argmax(z_d[0], axis=-1)
    x[2] = np.argmax(z_d[2], axis=-1)
    gamma = np.array([64, 64, 37], dtype=np.int32)
    for g in (None, gamma):
        got, ref = _run_verify(z_t, z_d, x, gamma=g, seed=5, step=9)
        H.assert_verify(got, ref, k)
        assert ref["n_accept"][0] == 64 and got["tokens"][0, 64] >= 0
        assert ref["n_accept"][2] == (64 if g is None else 37)
