"""The calls of a decode step (its four-call and its three-call form) captured into a HIP
graph (as a serving loop would run them) and replayed: every replay must reproduce the eager results.
The library enqueues kernels only - no allocation, no memset, no host sync -
so the whole step is capturable once each kernel has been launched eagerly."""
import numpy as np
import pytest
import torch

import svgen

import harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("form", ["four calls", "three calls"])
def test_step_replays_from_a_graph(form):
    P = H.sv()
    B, k, V = 8, 8, 32000
    cfgs = [svgen.make_config(1, B=B, k=k, V=V, dtype="bf16", seed=s) for s in (11, 12, 13)]
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = svgen.latency_table(B * k)
    d_es, d_ea, d_tab, d_lat = (H.dev(a) for a in (edges_s, edges_a, table, lat))
    f32 = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
    z_t = torch.zeros((B, k + 1, V), dtype=torch.bfloat16, device="cuda")
    z_d = torch.zeros((B, k, V), dtype=torch.bfloat16, device="cuda")
    z_c = torch.zeros((B, k, V), dtype=torch.bfloat16, device="cuda")
    x = i32(B, k)
    lse_d, lse_c, S, A, p_hat, ratio = (f32(B, k) for _ in range(6))
    gamma, offs, total = i32(B), i32(B + 1), i32(1)
    tokens, n_acc, flags = i32(B, k + 1), i32(B), i32(B)
    ws = P.alloc_workspace(B, k, V, P.SV_BF16)
    outs = (S, A, p_hat, gamma, offs, total, tokens, n_acc, flags, ratio)

    def step():
        P.sv_row_stats(z_d, z_c, x, lse_d, lse_c, S, A, None, None, ws)
        if form == "three calls":      # estimate + selection in one launch, draft normalisers handed over in ws
            P.sv_estimate_select(S, A, d_es, d_ea, d_tab, d_lat, P.SV_BATCH_GREEDY, p_hat, gamma, offs, total)
            P.sv_verify_sample_chained(z_t, None, z_d, x, gamma, 7, 3, tokens, n_acc, flags, ratio, ws)
            return
        P.sv_accept_estimate(S, A, d_es, d_ea, d_tab, p_hat, None)
        P.sv_select_length(p_hat, d_lat, P.SV_BATCH_GREEDY, gamma, offs, total)
        P.sv_verify_sample(z_t, None, z_d, x, gamma, 7, 3, tokens, n_acc, flags, ratio, ws)

    def load(c):
        z_t.copy_(c["z_t"]); z_d.copy_(c["z_d"]); z_c.copy_(c["z_c"]); x.copy_(c["x"])

    eager = []
    for c in cfgs:                                   # eager reference (also warms every kernel up)
        load(c)
        step()
        torch.cuda.synchronize()
        eager.append([o.clone() for o in outs])

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        load(cfgs[0])
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep in range(2):
        for c, ref in zip(cfgs, eager):
            load(c)
            for o in outs:
                o.fill_(-1)                          # stale results must not survive a replay
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for o, r in zip(outs, ref):
                assert np.array_equal(o.cpu().numpy(), r.cpu().numpy(), equal_nan=True)


def test_compacted_warped_step_replays_from_a_graph():
    """Same for the warped step on compacted supports (three compaction passes,
    sparse indicators, estimate, lengths, sparse verification)."""
    P = H.sv()
    B, k, V, cap = 8, 8, 32000, 64
    T, K, Pp = float(np.float32(0.7)), 20, 0.8
    cfgs = [svgen.make_config(1, B=B, k=k, V=V, dtype="bf16", seed=s) for s in (21, 22, 23)]
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = svgen.latency_table(B * k)
    d_es, d_ea, d_tab, d_lat = (H.dev(a) for a in (edges_s, edges_a, table, lat))
    f32 = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
    z_t = torch.zeros((B, k + 1, V), dtype=torch.bfloat16, device="cuda")
    z_d = torch.zeros((B, k, V), dtype=torch.bfloat16, device="cuda")
    z_c = torch.zeros((B, k, V), dtype=torch.bfloat16, device="cuda")
    x = i32(B, k)
    sup_t, sup_d, sup_c = P.Supports(B * (k + 1), cap), P.Supports(B * k, cap), P.Supports(B * k, cap)
    lse_d, lse_c, S, A, p_hat, ratio = (f32(B, k) for _ in range(6))
    gamma, offs, total = i32(B), i32(B + 1), i32(1)
    tokens, n_acc, flags = i32(B, k + 1), i32(B), i32(B)
    outs = (S, A, p_hat, gamma, offs, total, tokens, n_acc, flags, ratio, sup_t.count, sup_d.count, sup_c.count)

    def step():
        P.sv_warp_compact(z_t, T, K, Pp, sup_t)
        P.sv_warp_compact(z_d, T, K, Pp, sup_d)
        P.sv_warp_compact(z_c, T, K, Pp, sup_c)
        P.sv_row_stats_sparse(sup_d, sup_c, x, V, lse_d, lse_c, S, A)
        P.sv_accept_estimate(S, A, d_es, d_ea, d_tab, p_hat, None)
        P.sv_select_length(p_hat, d_lat, P.SV_BATCH_GREEDY, gamma, offs, total)
        P.sv_verify_sample_sparse(sup_t, None, sup_d, x, gamma, V, 7, 3, tokens, n_acc, flags, ratio)

    def load(c):
        z_t.copy_(c["z_t"]); z_d.copy_(c["z_d"]); z_c.copy_(c["z_c"]); x.copy_(c["x"])

    eager = []
    for c in cfgs:
        load(c)
        step()
        torch.cuda.synchronize()
        eager.append([o.clone() for o in outs])
        assert (sup_d.count > 0).all()

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        load(cfgs[0])
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep in range(2):
        for c, ref in zip(cfgs, eager):
            load(c)
            for o in outs:
                o.fill_(-1)
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for o, r in zip(outs, ref):
                assert np.array_equal(o.cpu().numpy(), r.cpu().numpy(), equal_nan=True)
