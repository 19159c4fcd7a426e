"""sv_repetition_penalty against the oracle: the penalised tensors must be identical bit for
bit (float32 arithmetic on both sides, bfloat16 rounded to nearest-even), dense and packed, with
duplicate and padded history entries, and with the drafted prefix."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O
from oracle import warp_oracle as W

import harness as H

pytestmark = pytest.mark.gpu


def _history(rng, B, n_hist, V):
    h = rng.integers(0, V, size=(B, n_hist)).astype(np.int32)
    if n_hist >= 4:
        h[:, 1] = h[:, 0]                       # duplicates: penalised once
        h[:, n_hist - 1] = -1                   # padding
        h[0, 2] = V                             # impossible ids are ignored
    return h


@pytest.mark.parametrize("B,k,V,dtype,n_hist,theta", [(2, 3, 1000, "f32", 17, 1.3), (3, 4, 32000, "bf16", 700, 1.1),
                                                      (2, 2, 152064, "bf16", 4000, 1.05), (1, 1, 7, "f32", 9, 2.0),
                                                      (4, 5, 4099, "bf16", 0, 1.2), (2, 8, 20011, "f32", 300, 0.8)])
def test_penalised_logits_are_identical_to_the_oracle(B, k, V, dtype, n_hist, theta):
    P = H.sv()
    rng = np.random.default_rng(B * 1000 + k)
    cfg = svgen.make_config(1, seed=4000 + V % 97, B=B, k=k, V=V, dtype=dtype, device="cuda")
    hist = _history(rng, B, n_hist, V) if n_hist else None
    x = cfg["x"].cpu().numpy()
    for name, with_x in (("z_t", True), ("z_d", True), ("z_c", False)):
        z = cfg[name].clone()
        if name == "z_d":
            z[0, 0, int(x[0, 0])] = 0.0          # zero stays zero, -inf stays -inf
            z[-1, -1, 1] = float("-inf")
        ref = W.repetition_penalty(svgen.to_numpy_bits(z), np.full((B, 1), -1) if hist is None else hist, theta,
                                   x=x if with_x else None)
        P.sv_repetition_penalty(z, None if hist is None else H.dev(hist, torch.int32), theta,
                                x=cfg["x"] if with_x else None)
        torch.cuda.synchronize()
        got = svgen.to_numpy_bits(z)
        same = got.view(np.uint32) == ref.view(np.uint32) if got.dtype == np.float32 else got == ref
        assert same.all(), (name, int((~same).sum()))
        if n_hist or with_x:
            assert not np.array_equal(got, svgen.to_numpy_bits(cfg[name]))       # something was penalised


def test_packed_target_rows_and_the_rest_of_the_step():
    """Packed target rows (lengths as the selection leaves them), then the penalised tensors go
    through the ordinary step: the oracle on the oracle's penalised logits gives the same."""
    P = H.sv()
    B, k, V = 5, 4, 32000
    rng = np.random.default_rng(5)
    cfg = svgen.make_config(1, seed=4321, B=B, k=k, V=V, dtype="bf16", device="cuda")
    hist = _history(rng, B, 64, V)
    gamma = np.array([4, 0, 2, 1, 3], dtype=np.int32)
    offs = np.concatenate([[0], np.cumsum(gamma + 1)]).astype(np.int32)
    packed = torch.cat([cfg["z_t"][b, :gamma[b] + 1] for b in range(B)]).contiguous()
    x = cfg["x"].cpu().numpy()
    theta = 1.15
    ref_t = W.repetition_penalty(svgen.to_numpy_bits(cfg["z_t"]), hist, theta, x=x)
    ref_d = W.repetition_penalty(svgen.to_numpy_bits(cfg["z_d"]), hist, theta, x=x)
    ref_c = W.repetition_penalty(svgen.to_numpy_bits(cfg["z_c"]), hist, theta, x=x)
    d_hist = H.dev(hist, torch.int32)
    P.sv_repetition_penalty(packed, d_hist, theta, x=cfg["x"], row_offsets=H.dev(offs, torch.int32), B=B,
                            rows_per_seq=k + 1)
    z_d, z_c = cfg["z_d"].clone(), cfg["z_c"].clone()
    P.sv_repetition_penalty(z_d, d_hist, theta, x=cfg["x"])
    P.sv_repetition_penalty(z_c, d_hist, theta, x=cfg["x"])
    torch.cuda.synchronize()
    got_packed = svgen.to_numpy_bits(packed)
    for b in range(B):
        for i in range(gamma[b] + 1):
            assert np.array_equal(got_packed[offs[b] + i], ref_t[b, i]), (b, i)
    assert np.array_equal(svgen.to_numpy_bits(z_d), ref_d) and np.array_equal(svgen.to_numpy_bits(z_c), ref_c)
    H.assert_row_stats(H.gpu_row_stats(z_d, z_c, cfg["x"]), O.row_stats(ref_d, ref_c, x))
    got = H.gpu_verify(packed, z_d, cfg["x"], gamma=gamma, t_offsets=offs, seed=2, step=9)
    H.assert_verify(got, H.oracle_verify(ref_t, ref_d, x, gamma=gamma, seed=2, step=9), k)


def test_three_tensors_in_one_launch_equal_three_launches():
    P = H.sv()
    B, k, V = 5, 4, 32000
    rng = np.random.default_rng(6)
    cfg = svgen.make_config(1, seed=4322, B=B, k=k, V=V, dtype="bf16", device="cuda")
    hist = H.dev(_history(rng, B, 200, V), torch.int32)
    gamma = np.array([4, 0, 2, 1, 3], dtype=np.int32)
    offs = H.dev(np.concatenate([[0], np.cumsum(gamma + 1)]).astype(np.int32), torch.int32)
    packed = torch.cat([cfg["z_t"][b, :gamma[b] + 1] for b in range(B)]).contiguous()
    one = [packed.clone(), cfg["z_d"].clone(), cfg["z_c"].clone()]
    P.sv_repetition_penalty(one[0], hist, 1.05, x=cfg["x"], row_offsets=offs, B=B, rows_per_seq=k + 1)
    P.sv_repetition_penalty(one[1], hist, 1.05, x=cfg["x"])
    P.sv_repetition_penalty(one[2], hist, 1.05, x=cfg["x"])
    many = [packed.clone(), cfg["z_d"].clone(), cfg["z_c"].clone()]
    P.sv_repetition_penalty_multi(many, hist, 1.05, x=cfg["x"], row_offsets=[offs, None, None], B=B,
                                  rows_per_seq=[k + 1, None, None])
    torch.cuda.synchronize()
    for a_, b_ in zip(one, many):
        assert torch.equal(a_.view(torch.int16), b_.view(torch.int16))
    assert not torch.equal(many[1].view(torch.int16), cfg["z_d"].view(torch.int16))


def test_limits_and_no_ops():
    P = H.sv()
    Bd = P.binding
    z = torch.zeros((2, 3, 100), dtype=torch.float32, device="cuda")
    h = torch.zeros((2, 5), dtype=torch.int32, device="cuda")
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(P.SvError) as e:
            P.sv_repetition_penalty(z, h, bad)
        assert e.value.status == Bd.SV_ERR_INVALID_ARG
    big = torch.zeros((2, 4097), dtype=torch.int32, device="cuda")
    with pytest.raises(P.SvError) as e:
        P.sv_repetition_penalty(z, big, 1.2)
    assert e.value.status == Bd.SV_ERR_TOO_LARGE
    z[:] = 2.0
    P.sv_repetition_penalty(z, h, 1.0)                        # theta = 1: nothing changes
    torch.cuda.synchronize()
    assert (z == 2.0).all()
    P.sv_repetition_penalty(z, h, 2.0)                        # token 0 of every row halves, once
    torch.cuda.synchronize()
    assert (z[:, :, 0] == 1.0).all() and (z[:, :, 1:] == 2.0).all()
