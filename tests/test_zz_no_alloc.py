"""The entry point that allocates nothing (sv_verify_sample_static: library-held
device scratch instead of a caller workspace) against sv_verify_sample on the
same inputs: two calls in a row, the second on a smaller input, so that whatever
the first call left in the shared scratch is seen not to matter.  Integers are
compared bit for bit, the ratios to the last bit as well (same kernels)."""
import ctypes

import numpy as np
import pytest
import torch

import svgen

pytestmark = pytest.mark.gpu


def _outputs(B, k):
    return dict(tokens=torch.full((B, k + 1), -5, dtype=torch.int32, device="cuda"),
                n_accept=torch.full((B,), -5, dtype=torch.int32, device="cuda"),
                flags=torch.full((B,), 0x7FFF, dtype=torch.int32, device="cuda"),
                ratio=torch.full((B, k), -5.0, dtype=torch.float32, device="cuda"))


def _run_pair(P, cfg, gamma, seed, step):
    z_t, z_d, x = cfg["z_t"].cuda(), cfg["z_d"].cuda(), cfg["x"].cuda()
    B, k, V = z_d.shape
    g = None if gamma is None else torch.as_tensor(gamma, dtype=torch.int32).cuda()
    ref, got = _outputs(B, k), _outputs(B, k)
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(z_d))
    P.sv_verify_sample(z_t, None, z_d, x, g, seed, step, ref["tokens"], ref["n_accept"], ref["flags"],
                       ref["ratio"], ws)
    torch.cuda.synchronize()
    # the call under test: no workspace, and no allocation inside it
    before = torch.cuda.memory_allocated()
    P.sv_verify_sample_static(z_t, None, z_d, x, g, seed, step, got["tokens"], got["n_accept"], got["flags"],
                              got["ratio"])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name in ref:
        a, b = ref[name].cpu().numpy(), got[name].cpu().numpy()
        if name == "ratio":
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), name
        else:
            assert np.array_equal(a, b), (name, a, b)
    return ref


def test_static_scratch_entry_point_matches_workspace_entry_point():
    import paper_2509_24328_amd as P
    big = svgen.make_config(1, B=6, k=5, V=40000, dtype="bf16", seed=4242)
    r1 = _run_pair(P, big, None, seed=11, step=3)
    assert (r1["n_accept"].cpu().numpy() >= 0).all()
    # second call: fewer sequences, shorter drafts, smaller vocabulary, ragged lengths, fp32
    small = svgen.make_config(0, B=3, k=2, V=5000, dtype="f32", seed=4243)
    r2 = _run_pair(P, small, [2, 0, 1], seed=11, step=4)
    assert (r2["tokens"].cpu().numpy()[:, 0] >= 0).all()


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import paper_2509_24328_amd as P
    from paper_2509_24328_amd import binding as Bd
    p = ctypes.c_void_p(256 * 1024)          # never dereferenced: the size check comes first
    B, k, V = 4096, 64, 152064
    assert P.sv_workspace_bytes(B, k, V, P.SV_BF16) > Bd.SV_STATIC_SCRATCH_BYTES
    rc = Bd.lib.sv_verify_sample_static(p, None, 0, p, p, None, B, k, V, Bd.SV_BF16, 0, 0, p, p, p, None, None)
    assert rc == Bd.SV_ERR_TOO_LARGE
    assert "TOO_LARGE" in P.sv_strerror(rc)
