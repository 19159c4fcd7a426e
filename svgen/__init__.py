"""Seeded synthetic inputs for the SV hot path.

This module holds none of the method's arithmetic: it only draws logits,
drafted tokens, a profile table and a latency table with fixed seeds, so that
the CPU oracle and the HIP path can be fed the same stored values.  It is the
only module both sides' tests share.

The logits stand in for the outputs of the draft / companion / target models
of the paper's evaluation (target vocabularies of its 13B-72B model families:
32 000, 128 256 and 152 064 entries); the paper's datasets and checkpoints are
not used.  Recipes (generator seed = 1000 + config index unless given):

  0: B=1  k=4  V=32000  fp32  z_t ~ N(0, 2^2); z_d = z_t + N(0,1); z_c = z_t + N(0,1) indep.
  1: B=8  k=8  V=32000  bf16  z_t ~ N(0, 2^2); sigma per row from {0.5,1,2,4};
                              z_d = z_t + sigma n_d; z_c = z_t + sigma (0.5 n_d + sqrt(.75) n')
  2: B=32 k=8  V=128256 bf16  z_t = 3 * Student-t(nu=3); sigma ~ U[0.5,3] per sequence;
                              z_d, z_c = z_t + independent N(0, sigma^2)
  3: B=64 k=8  V=152064 bf16  z_t ~ N(0, 2.5^2), 1% of entries +8; sigma per sequence
                              from {0.5,1,2,4,8}; z_d, z_c as in 2          (headline)
  4: B=64 k=16 V=152064 bf16  as 3 with sigma ~ U[0.25,6] per sequence (ragged verification)

Values are drawn in float32, rounded once (round-to-nearest-even) to the
storage dtype; drafted tokens are drawn from softmax of the stored draft row.
"""
from __future__ import annotations

import math

import numpy as np
import torch

CONFIGS = [
    dict(name="cfg1_B1_k4_V32000_f32", B=1, k=4, V=32000, dtype="f32"),
    dict(name="cfg2_B8_k8_V32000_bf16", B=8, k=8, V=32000, dtype="bf16"),
    dict(name="cfg3_B32_k8_V128256_bf16", B=32, k=8, V=128256, dtype="bf16"),
    dict(name="cfg4_B64_k8_V152064_bf16", B=64, k=8, V=152064, dtype="bf16"),
    dict(name="cfg5_B64_k16_V152064_bf16_ragged", B=64, k=16, V=152064, dtype="bf16"),
]

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _rand(shape, g, device):
    return torch.rand(shape, generator=g, device=device, dtype=torch.float32)


def _choice(values, n, g, device):
    idx = torch.randint(0, len(values), (n,), generator=g, device=device)
    return torch.tensor(values, dtype=torch.float32, device=device)[idx]


def make_config(index, seed=None, B=None, k=None, V=None, dtype=None, device="cpu"):
    """Draw the inputs of config `index` (0-based), optionally at other sizes.

    Returns dict with torch tensors on `device`:
      z_t [B, k+1, V], z_d [B, k, V], z_c [B, k, V] (storage dtype), x [B, k] int32,
    plus the sizes and dtype tag.  Generation is sequence by sequence so that
    peak host memory stays near one sequence's float32 block.
    """
    cfg = CONFIGS[index]
    B = cfg["B"] if B is None else B
    k = cfg["k"] if k is None else k
    V = cfg["V"] if V is None else V
    dtype = cfg["dtype"] if dtype is None else dtype
    tdt = _TORCH_DTYPE[dtype]
    seed = 1000 + index if seed is None else seed
    g = torch.Generator(device=device)
    g.manual_seed(seed)

    z_t = torch.empty((B, k + 1, V), dtype=tdt, device=device)
    z_d = torch.empty((B, k, V), dtype=tdt, device=device)
    z_c = torch.empty((B, k, V), dtype=tdt, device=device)
    x = torch.empty((B, k), dtype=torch.int32, device=device)

    # per-sequence / per-row noise scales, drawn up front
    if index == 0:
        sigma = torch.ones((B, k), device=device)
    elif index == 1:
        sigma = _choice([0.5, 1.0, 2.0, 4.0], B * k, g, device).reshape(B, k)
    elif index == 2:
        sigma = (0.5 + 2.5 * _rand((B,), g, device))[:, None].expand(B, k)
    elif index == 3:
        sigma = _choice([0.5, 1.0, 2.0, 4.0, 8.0], B, g, device)[:, None].expand(B, k)
    elif index == 4:
        sigma = (0.25 + 5.75 * _rand((B,), g, device))[:, None].expand(B, k)
    else:
        raise IndexError(index)

    for b in range(B):
        if index in (0, 1):
            t = 2.0 * _randn((k + 1, V), g, device)
        elif index == 2:
            n0 = _randn((k + 1, V), g, device)
            chi = (_randn((3, k + 1, V), g, device) ** 2).sum(0) / 3.0
            t = 3.0 * n0 / torch.sqrt(chi)
        else:
            t = 2.5 * _randn((k + 1, V), g, device)
            t = t + 8.0 * (_rand((k + 1, V), g, device) < 0.01).float()
        n_d = _randn((k, V), g, device)
        n_c = _randn((k, V), g, device)
        sg = sigma[b][:, None]
        d = t[:k] + sg * n_d
        if index == 1:
            c = t[:k] + sg * (0.5 * n_d + math.sqrt(0.75) * n_c)
        else:
            c = t[:k] + sg * n_c
        z_t[b] = t.to(tdt)
        z_d[b] = d.to(tdt)
        z_c[b] = c.to(tdt)
        p = torch.softmax(z_d[b].float(), dim=-1)
        x[b] = torch.multinomial(p, 1, generator=g).squeeze(-1).to(torch.int32)
    return dict(z_t=z_t, z_d=z_d, z_c=z_c, x=x, B=B, k=k, V=V, dtype=dtype,
                name=cfg["name"], seed=seed, sigma=sigma)


def make_near_pairs(B, V, dtype, seed, lo, hi, device="cpu"):
    """Target / draft rows that differ by very little, one drafted position per
    sequence, with a rejection forced at it: inputs for checks of the residual
    draw at small residual mass.

    z_t [B, 2, V] ~ N(0, 2.5^2) (row 1 = bonus row); z_d [B, 1, V] differs from
    z_t[:, 0] by a per-sequence amount d_b, log-uniform in [lo, hi]:
      f32 : z_d = z_t + d_b * N(0, 1)  (rounded to float32)
      bf16: a random fraction min(1, d_b) of the entries moved by one bfloat16 ulp,
            up or down with equal probability (bfloat16 has no finer step)
    The drafted token x[b, 0] is a random id whose logit is set to -inf in both
    rows: its acceptance ratio is 0/0 and it is rejected, so position 0 is
    always drawn from the residual.  Returns dict(z_t, z_d, x, d).
    """
    tdt = _TORCH_DTYPE[dtype]
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    z_t = torch.empty((B, 2, V), dtype=tdt, device=device)
    z_d = torch.empty((B, 1, V), dtype=tdt, device=device)
    u = _rand((B,), g, device)
    d = torch.exp(math.log(lo) + u * (math.log(hi) - math.log(lo)))
    x = torch.randint(0, V, (B, 1), generator=g, device=device).to(torch.int32)
    for b in range(B):
        t = (2.5 * _randn((2, V), g, device)).to(tdt)
        if dtype == "f32":
            dr = (t[0] + d[b] * _randn((V,), g, device)).to(tdt)
        else:
            move = _rand((V,), g, device) < d[b]
            up = _rand((V,), g, device) < 0.5
            bits = t[0].view(torch.int16).to(torch.int32)
            step = torch.where(up, 1, -1) * move.to(torch.int32)
            # one ulp away from zero / towards zero in sign-magnitude order; values near 0 and
            # the largest finite magnitudes stay as they are
            mag = bits & 0x7FFF
            ok = (mag > 0x0080) & (mag < 0x7F00)
            new_mag = torch.where(ok, mag + step, mag)
            dr = ((bits & 0x8000) | new_mag).to(torch.int16).view(torch.bfloat16)
        tok = int(x[b, 0])
        t[0, tok] = float("-inf")
        dr[tok] = float("-inf")
        z_t[b] = t
        z_d[b, 0] = dr
    return dict(z_t=z_t, z_d=z_d, x=x, d=d)


def profile_table(n_s=10, n_a=10):
    """A closed-form, monotone stand-in for the profiled acceptance table.

    Uniform edges on [0,1] in both S and A; cell value
    clip(0.05 + 0.9 (0.5 s_mid + 0.5 a_mid), 0, 1).  The paper builds its table
    from 512 profiled samples of real models, which are not available here.
    Returns float32 (edges_s [n_s+1], edges_a [n_a+1], table [n_s, n_a]).
    """
    edges_s = np.linspace(0.0, 1.0, n_s + 1).astype(np.float32)
    edges_a = np.linspace(0.0, 1.0, n_a + 1).astype(np.float32)
    s_mid = 0.5 * (edges_s[:-1] + edges_s[1:]).astype(np.float64)
    a_mid = 0.5 * (edges_a[:-1] + edges_a[1:]).astype(np.float64)
    table = np.clip(0.05 + 0.9 * (0.5 * s_mid[:, None] + 0.5 * a_mid[None, :]), 0.0, 1.0)
    return edges_s, edges_a, table.astype(np.float32)


def latency_table(n, t0=30.0, d=0.08, m0=128):
    """latency[M], M = 0..n: t0 + sum_{m<M} d * min(1, (m+1)/m0).

    Increments grow up to m0 verified tokens and stay constant afterwards, the
    shape the paper's latency assumption describes; the numbers themselves are
    arbitrary (the paper prints none).
    """
    inc = d * np.minimum(1.0, (np.arange(n, dtype=np.float64) + 1.0) / m0)
    lat = t0 + np.concatenate(([0.0], np.cumsum(inc)))
    return lat.astype(np.float32)


def to_numpy_bits(t):
    """Stored logits as the NumPy array the oracle takes: float32 as is,
    bfloat16 as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def checksum(t):
    """Order-dependent 64-bit checksum of a tensor's bytes (for logging)."""
    a = to_numpy_bits(t).reshape(-1).view(np.uint8)
    pad = (-a.size) % 8
    if pad:
        a = np.concatenate([a, np.zeros(pad, dtype=np.uint8)])
    w = a.view(np.uint64)
    mult = np.arange(1, w.size + 1, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
    return int(np.bitwise_xor.reduce(w * mult))
