"""CPU-only checks of the boundary: the library loads, exports every symbol
the header declares, and rejects bad arguments on the host (no launch)."""
import ctypes
import os
import re

import paper_2509_24328_amd as P
from paper_2509_24328_amd import binding as Bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "sv.h")).read()
    declared = set(re.findall(r"\b(sv_[a-z_]+)\s*\(", header))
    assert declared == set(Bd.EXPORTS)
    for name in declared:
        assert getattr(Bd.lib, name) is not None


def test_status_strings():
    for code in range(-7, 1):
        assert P.sv_strerror(code).startswith("SV_")
    assert "unknown" in P.sv_strerror(-99)


def test_workspace_sizing():
    assert P.sv_workspace_bytes(64, 8, 152064, P.SV_BF16) > 0
    assert P.sv_workspace_bytes(64, 8, 152064, P.SV_BF16) % 256 == 0
    assert P.sv_workspace_bytes(64, 0, 152064, P.SV_BF16) == 0
    assert P.sv_workspace_bytes(64, 8, 152064, 7) == 0
    assert P.sv_workspace_bytes(128, 8, 1000, P.SV_F32) > P.sv_workspace_bytes(64, 8, 1000, P.SV_F32)


def test_argument_errors_are_reported_before_any_launch():
    L = Bd.lib
    p = ctypes.c_void_p(256 * 1024)          # a non-NULL, aligned, never dereferenced address
    odd = ctypes.c_void_p(256 * 1024 + 1)
    big = 1 << 30
    rs = lambda **kw: L.sv_row_stats(kw.get("zd", p), p, p, kw.get("B", 2), kw.get("k", 2),
                                     kw.get("V", 8), kw.get("dt", 1), p, p, p, p, None, None, None, None,
                                     kw.get("ws", p), kw.get("wsb", big), None)
    assert rs(dt=3) == Bd.SV_ERR_DTYPE
    assert rs(k=0) == Bd.SV_ERR_INVALID_ARG
    assert rs(V=0) == Bd.SV_ERR_INVALID_ARG
    assert rs(B=-1) == Bd.SV_ERR_INVALID_ARG
    assert rs(zd=None) == Bd.SV_ERR_NULL
    assert rs(zd=odd) == Bd.SV_ERR_ALIGN
    assert rs(ws=None) == Bd.SV_ERR_WORKSPACE
    assert rs(wsb=16) == Bd.SV_ERR_WORKSPACE
    assert rs(ws=odd) == Bd.SV_ERR_WORKSPACE

    vs = lambda **kw: L.sv_verify_sample(kw.get("zt", p), kw.get("offs", None), kw.get("nt", 0), p, p,
                                         None, kw.get("B", 2), kw.get("k", 2), 8, kw.get("dt", 1), 0, 0,
                                         kw.get("out", p), p, p, None, kw.get("ws", p),
                                         kw.get("wsb", big), None)
    assert vs(dt=-1) == Bd.SV_ERR_DTYPE
    assert vs(k=65) == Bd.SV_ERR_TOO_LARGE
    assert vs(zt=None) == Bd.SV_ERR_NULL
    assert vs(out=None) == Bd.SV_ERR_NULL
    assert vs(offs=p, nt=-1) == Bd.SV_ERR_INVALID_ARG
    assert vs(wsb=0) == Bd.SV_ERR_WORKSPACE

    vc = lambda **kw: L.sv_verify_sample_chained(kw.get("zt", p), None, 0, p, p, None, kw.get("B", 2),
                                                 kw.get("k", 2), 8, kw.get("dt", 1), 0, 0, p, p, p, None,
                                                 kw.get("ws", p), kw.get("wsb", big), None)
    assert vc(dt=-1) == Bd.SV_ERR_DTYPE
    assert vc(k=65) == Bd.SV_ERR_TOO_LARGE
    assert vc(zt=None) == Bd.SV_ERR_NULL
    assert vc(ws=None) == Bd.SV_ERR_WORKSPACE
    assert vc(B=0) == Bd.SV_OK

    ae = lambda **kw: L.sv_accept_estimate(kw.get("S", p), p, kw.get("n", 4), p, kw.get("ns", 5), p, 5,
                                           p, p, None, None)
    assert ae(n=-1) == Bd.SV_ERR_INVALID_ARG
    assert ae(ns=0) == Bd.SV_ERR_INVALID_ARG
    assert ae(S=None) == Bd.SV_ERR_NULL
    assert ae(S=odd) == Bd.SV_ERR_ALIGN

    sl = lambda **kw: L.sv_select_length(kw.get("p", p), kw.get("B", 4), kw.get("k", 4), p,
                                         kw.get("nl", 17), kw.get("mode", 0), p, p, p, None)
    assert sl(mode=2) == Bd.SV_ERR_INVALID_ARG
    assert sl(nl=16) == Bd.SV_ERR_INVALID_ARG
    assert sl(B=Bd.SV_SELECT_MAX_KEYS + 1, k=1, nl=10000) == Bd.SV_ERR_TOO_LARGE
    assert sl(p=None) == Bd.SV_ERR_NULL
    assert sl(B=0) == Bd.SV_OK and sl(B=0, p=None) == Bd.SV_OK      # empty batch: nothing to do, as in the other calls
    assert sl(B=-1) == Bd.SV_ERR_INVALID_ARG


def test_profile_pass_argument_errors():
    L = Bd.lib
    p = ctypes.c_void_p(256 * 1024)
    odd = ctypes.c_void_p(256 * 1024 + 1)
    big = 1 << 30
    ar = lambda **kw: L.sv_accept_ratio(kw.get("zt", p), kw.get("tr", 3), p, p, 2, kw.get("k", 2), 8,
                                        kw.get("dt", 1), kw.get("ratio", p), None, kw.get("ws", p), big, None)
    assert ar(dt=9) == Bd.SV_ERR_DTYPE
    assert ar(tr=5) == Bd.SV_ERR_INVALID_ARG
    assert ar(zt=None) == Bd.SV_ERR_NULL
    assert ar(ratio=odd) == Bd.SV_ERR_ALIGN
    assert ar(ws=None) == Bd.SV_ERR_WORKSPACE
    qe = lambda **kw: L.sv_quantile_edges(kw.get("v", p), kw.get("n", 10), kw.get("nb", 4),
                                          ctypes.c_float(0), ctypes.c_float(1), kw.get("e", p), None)
    assert qe(n=-1) == Bd.SV_ERR_INVALID_ARG
    assert qe(nb=0) == Bd.SV_ERR_INVALID_ARG
    assert qe(n=8193) == Bd.SV_ERR_TOO_LARGE
    assert qe(e=None) == Bd.SV_ERR_NULL
    assert qe(v=None) == Bd.SV_ERR_NULL
    pa = lambda **kw: L.sv_profile_accumulate(kw.get("S", p), p, p, kw.get("n", 4), p, 5, p, 5,
                                              kw.get("nx", 10), p, kw.get("sx", p), None)
    assert pa(n=-2) == Bd.SV_ERR_INVALID_ARG
    assert pa(nx=0) == Bd.SV_ERR_INVALID_ARG
    assert pa(nx=2000) == Bd.SV_ERR_TOO_LARGE
    assert pa(S=None) == Bd.SV_ERR_NULL
    assert pa(sx=ctypes.c_void_p(256 * 1024 + 4)) == Bd.SV_ERR_ALIGN
    pf = lambda **kw: L.sv_profile_finalize(kw.get("c", p), p, kw.get("ns", 5), 5, kw.get("nx", 10), p,
                                            kw.get("info", p), None)
    assert pf(ns=0) == Bd.SV_ERR_INVALID_ARG
    assert pf(nx=1025) == Bd.SV_ERR_TOO_LARGE
    assert pf(c=None) == Bd.SV_ERR_NULL
    assert pf(info=ctypes.c_void_p(256 * 1024 + 4)) == Bd.SV_ERR_ALIGN


def test_warp_cutoffs_argument_errors():
    L = Bd.lib
    p = ctypes.c_void_p(256 * 1024)
    f = ctypes.c_float
    wc = lambda **kw: L.sv_warp_cutoffs(kw.get("z", p), kw.get("rows", 4), kw.get("V", 8), kw.get("dt", 1),
                                        f(kw.get("T", 0.7)), 20, f(kw.get("P", 0.8)), kw.get("cut", p), None, None)
    assert wc(dt=2) == Bd.SV_ERR_DTYPE
    assert wc(T=0.0) == Bd.SV_ERR_INVALID_ARG
    assert wc(P=0.0) == Bd.SV_ERR_INVALID_ARG
    assert wc(V=0) == Bd.SV_ERR_INVALID_ARG
    assert wc(z=None) == Bd.SV_ERR_NULL
    assert wc(cut=ctypes.c_void_p(256 * 1024 + 2)) == Bd.SV_ERR_ALIGN
    assert wc(rows=0) == Bd.SV_OK


def test_warped_entry_points_reject_bad_temperatures():
    L = Bd.lib
    p = ctypes.c_void_p(256 * 1024)
    f = ctypes.c_float
    rs = lambda Td, Tc, dt=1: L.sv_row_stats_warped(p, p, p, 2, 2, 64, dt, f(Td), None, f(Tc), None,
                                                    p, p, p, p, None, None, None, None, p, 1 << 20, None)
    vs = lambda Tt, Td, dt=1: L.sv_verify_sample_warped(p, None, 0, p, p, None, 2, 2, 64, dt, f(Tt), None,
                                                        f(Td), None, 1, 0, p, p, p, None, p, 1 << 20, None)
    for call in (rs, vs):
        assert call(0.0, 1.0) == Bd.SV_ERR_INVALID_ARG
        assert call(1.0, -1.0) == Bd.SV_ERR_INVALID_ARG
        assert call(float("nan"), 1.0) == Bd.SV_ERR_INVALID_ARG
        assert call(1.0, 1e4) == Bd.SV_ERR_INVALID_ARG
        assert call(1.0, 1.0, dt=7) == Bd.SV_ERR_DTYPE
    # a misaligned cutoff array is refused before anything is launched
    bad = ctypes.c_void_p(256 * 1024 + 2)
    assert L.sv_row_stats_warped(p, p, p, 2, 2, 64, 1, f(1.0), bad, f(1.0), None, p, p, p, p, None, None, None,
                                 None, p, 1 << 20, None) == Bd.SV_ERR_ALIGN
    assert L.sv_verify_sample_warped(p, None, 0, p, p, None, 2, 2, 64, 1, f(1.0), None, f(1.0), bad, 1, 0, p, p,
                                     p, None, p, 1 << 20, None) == Bd.SV_ERR_ALIGN


def test_compact_and_sparse_argument_errors():
    L = Bd.lib
    p = ctypes.c_void_p(256 * 1024)
    odd = ctypes.c_void_p(256 * 1024 + 4)
    f = ctypes.c_float
    wc = lambda **kw: L.sv_warp_compact(kw.get("z", p), kw.get("rows", 4), 8, kw.get("dt", 1), f(kw.get("T", 0.7)), 20,
                                        f(0.8), kw.get("cap", 64), kw.get("count", p), p, kw.get("prob", p), p,
                                        None, None, None)
    assert wc(cap=0) == Bd.SV_ERR_INVALID_ARG
    assert wc(cap=Bd.SV_SUPPORT_MAX_CAP + 1) == Bd.SV_ERR_INVALID_ARG
    assert wc(T=0.0) == Bd.SV_ERR_INVALID_ARG
    assert wc(dt=3) == Bd.SV_ERR_DTYPE
    assert wc(count=None) == Bd.SV_ERR_NULL
    assert wc(prob=odd) == Bd.SV_ERR_ALIGN
    assert wc(rows=0) == Bd.SV_OK
    rs = lambda **kw: L.sv_row_stats_sparse(p, p, kw.get("prob", p), p, p, p, p, p, kw.get("cap", 64), kw.get("x", p),
                                            kw.get("B", 2), 2, 100, p, p, p, p, None, None, None, None, None)
    assert rs(cap=0) == Bd.SV_ERR_INVALID_ARG
    assert rs(x=None) == Bd.SV_ERR_NULL
    assert rs(prob=odd) == Bd.SV_ERR_ALIGN
    assert rs(B=0) == Bd.SV_OK
    vs = lambda **kw: L.sv_verify_sample_sparse(p, p, kw.get("prob", p), None, 0, p, p, p, kw.get("cap", 64), p, None,
                                                kw.get("B", 2), kw.get("k", 2), 100, 1, 0, kw.get("out", p), p, p,
                                                None, None)
    assert vs(cap=2000) == Bd.SV_ERR_INVALID_ARG
    assert vs(k=Bd.SV_MAX_K + 1) == Bd.SV_ERR_TOO_LARGE
    assert vs(out=None) == Bd.SV_ERR_NULL
    assert vs(prob=odd) == Bd.SV_ERR_ALIGN
    assert vs(B=0) == Bd.SV_OK


def test_binding_refuses_host_and_strided_tensors():
    import pytest
    import torch
    with pytest.raises(ValueError):
        Bd._ptr(torch.zeros(4))                    # host memory
    assert Bd._ptr(None) is None


def test_uniforms_argument_errors():
    L = Bd.lib
    p = ctypes.c_void_p(256 * 1024)
    assert L.sv_uniforms(1, 0, 4, 0, p, p, None) == Bd.SV_ERR_INVALID_ARG
    assert L.sv_uniforms(1, 0, 4, 4, None, p, None) == Bd.SV_ERR_NULL
    assert L.sv_uniforms(1, 0, 4, 4, ctypes.c_void_p(256 * 1024 + 4), p, None) == Bd.SV_ERR_ALIGN
    assert L.sv_uniforms(1, 0, 0, 4, None, None, None) == Bd.SV_OK


def test_accept_ratio_sparse_argument_errors():
    L = Bd.lib
    p = ctypes.c_void_p(256 * 1024)
    call = lambda **kw: L.sv_accept_ratio_sparse(p, p, p, kw.get("tr", 3), p, p, p, kw.get("cap", 64), kw.get("x", p),
                                                 kw.get("B", 2), 2, 100, kw.get("ratio", p), None, None)
    assert call(tr=5) == Bd.SV_ERR_INVALID_ARG
    assert call(cap=0) == Bd.SV_ERR_INVALID_ARG
    assert call(x=None) == Bd.SV_ERR_NULL
    assert call(ratio=ctypes.c_void_p(256 * 1024 + 2)) == Bd.SV_ERR_ALIGN
    assert call(B=0) == Bd.SV_OK
