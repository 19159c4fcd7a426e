"""Tensors beyond 2^31 elements and 2^32 bytes: B = 1024, k = 16, V = 152064 in bfloat16 is
16384 draft rows of 304128 bytes (4.98 GB per tensor), so row and byte offsets that fit 32 bits
at the benchmark sizes no longer do.  Inputs are drawn on the GPU (simple recipe: the test is
about addressing); the oracle checks the sequences at the start, on both sides of the 4 GiB
boundary and at the end, each handed over with the Philox uniforms of its own batch index."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu

B, K, V = 1024, 16, 152064


def _inputs():
    g = torch.Generator(device="cuda")
    g.manual_seed(20250924)
    z_t = torch.empty((B, K + 1, V), dtype=torch.bfloat16, device="cuda")
    z_d = torch.empty((B, K, V), dtype=torch.bfloat16, device="cuda")
    z_c = torch.empty((B, K, V), dtype=torch.bfloat16, device="cuda")
    step = 64
    for b0 in range(0, B, step):                                     # 64 sequences (0.66 GB of float32) at a time
        t = torch.randn((step, K + 1, V), generator=g, device="cuda") * 2.5
        z_t[b0:b0 + step] = t.to(torch.bfloat16)
        z_d[b0:b0 + step] = (t[:, :K] + torch.randn((step, K, V), generator=g, device="cuda")).to(torch.bfloat16)
        z_c[b0:b0 + step] = (t[:, :K] + torch.randn((step, K, V), generator=g, device="cuda")).to(torch.bfloat16)
        del t
    x = torch.argmax(z_d[:, :, :4096].float() + torch.rand((B, K, 4096), generator=g, device="cuda") * 6, dim=2)
    return z_t, z_d, z_c, x.to(torch.int32).contiguous()


def test_row_and_byte_offsets_beyond_32_bits():
    P = H.sv()
    assert B * K * V > 2 ** 31 and B * K * V * 2 > 2 ** 32
    z_t, z_d, z_c, x = _inputs()
    ws = P.alloc_workspace(B, K, V, P.SV_BF16)
    f32 = lambda: torch.full((B, K), -7.0, dtype=torch.float32, device="cuda")
    lse_d, lse_c, S, A, pdx = f32(), f32(), f32(), f32(), f32()
    fl = torch.full((B, K), 0xFFFF, dtype=torch.int32, device="cuda")
    P.sv_row_stats(z_d, z_c, x, lse_d, lse_c, S, A, None, fl, ws, pd_x=pdx)
    out = {}
    for name, call in (("plain", P.sv_verify_sample), ("chained", P.sv_verify_sample_chained)):
        tok = torch.full((B, K + 1), -5, dtype=torch.int32, device="cuda")
        n_acc = torch.full((B,), -5, dtype=torch.int32, device="cuda")
        flags = torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda")
        ratio = torch.full((B, K), -5.0, dtype=torch.float32, device="cuda")
        call(z_t, None, z_d, x, None, 9, 4, tok, n_acc, flags, ratio, ws)
        torch.cuda.synchronize()
        out[name] = dict(tokens=tok.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
                         flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
    stats = dict(lse_d=lse_d.cpu().numpy(), lse_c=lse_c.cpu().numpy(), S=S.cpu().numpy(), A=A.cpu().numpy(),
                 pd_x=pdx.cpu().numpy(), flags=fl.cpu().numpy())
    # the row whose bytes straddle 4 GiB, in the draft tensor and in the target tensor
    row_d = (2 ** 32) // (V * 2)
    picks = sorted({0, row_d // K - 1, row_d // K, row_d // K + 1, (2 ** 32) // (V * 2 * (K + 1)), B // 2, B - 1})
    for b in picks:
        zt, zd, zc = (svgen.to_numpy_bits(t[b:b + 1].cpu()) for t in (z_t, z_d, z_c))
        xb = x[b:b + 1].cpu().numpy()
        ref = O.row_stats(zd, zc, xb)
        got = {n: v[b:b + 1] for n, v in stats.items()}
        H.assert_row_stats(got, ref, with_kl=False)
        refv = H.oracle_verify(zt, zd, xb, seed=9, step=4, uniforms=H.uniforms_of([b], K, seed=9, step=4))
        for name in out:
            H.assert_verify({n: v[b:b + 1] for n, v in out[name].items()}, refv, K)
    # every sequence: the two verification paths agree, no flag that says a row was unusable
    soft = O.FLAG_NEAR_TIE | O.FLAG_NEAR_CDF_EDGE
    clear = ((out["plain"]["flags"] | out["chained"]["flags"]) & soft) == 0
    # (these rows are nearly flat: a token holds about 1e-5 of the mass, so the absolute part of the
    # near-edge band, 1e-6, covers a good share of every interval and many draws are flagged)
    assert clear.sum() > B // 2
    for name in ("tokens", "n_accept", "flags"):
        assert np.array_equal(out["plain"][name][clear], out["chained"][name][clear]), name
    assert ((out["plain"]["flags"] & (O.FLAG_BAD_ROW | O.FLAG_BAD_TOKEN)) == 0).all()
    assert (stats["flags"] == 0).all() and np.isfinite(stats["S"]).all()
    assert (out["plain"]["tokens"][:, 0] >= 0).all()
