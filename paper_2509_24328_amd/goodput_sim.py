"""Step-level goodput simulation of SV against plain speculative decoding on
synthetic logits, entirely through the C ABI.

What the paper measures end to end with real models (goodput = accepted tokens
per unit time, Sec. 5 and Sec. 7.2) is modelled here per decode step:

  * profile:  P(T | S, A) is built on a held-out batch (distinct seed) with the
              profile pass (sv_row_stats, sv_accept_ratio, sv_profile_accumulate,
              sv_profile_finalize), as the paper builds it from profiled samples;
  * SD step:  every sequence verifies all k drafted tokens;
  * SV step:  sv_row_stats -> sv_accept_estimate -> sv_select_length picks the
              lengths, only those positions are verified;
  * cost:     latency[M] of the caller's latency table, M = drafted tokens sent to
              the target in the step (the paper's profiled verification latency).

Goodput of a run = accepted drafted tokens / sum of step latencies; the accept
rate is accepted / verified.  Only the qualitative picture can be compared with
the paper (its numbers need its models and hardware): SV trades a little
acceptance volume for much less verification work where drafts are poor.

With --temperature / --top-k / --top-p the whole simulation runs on the warped
distributions the paper's experiments sample from (appendix table of sampling
hyper-parameters), through the compacted-support calls: sv_warp_compact once per
logit tensor, then sv_row_stats_sparse, sv_accept_ratio_sparse (profile) and
sv_verify_sample_sparse.

Run:  python -m paper_2509_24328_amd.goodput_sim [--config 1] [--steps 20]
      python -m paper_2509_24328_amd.goodput_sim --temperature 0.7 --top-k 20 --top-p 0.8
"""
from __future__ import annotations

import argparse
import json

import numpy as np
import torch

from . import binding as B_
from .binding import (SV_BATCH_GREEDY, Supports, alloc_workspace, sv_accept_estimate, sv_accept_ratio,
                      sv_accept_ratio_sparse, sv_profile_accumulate, sv_profile_finalize, sv_row_stats,
                      sv_row_stats_sparse, sv_select_length, sv_verify_sample, sv_verify_sample_sparse,
                      sv_warp_compact)

SUPPORT_CAP = 256


def _compact(batch, warp):
    """Supports of the three warped tensors of a batch; raises if a row does not fit."""
    T, K, Pp = warp
    sups = {}
    for name in ("z_t", "z_d", "z_c"):
        z = batch[name]
        sup = Supports(z.shape[0] * z.shape[1], SUPPORT_CAP)
        sv_warp_compact(z, T, K, Pp, sup)
        sups[name] = sup
    torch.cuda.synchronize()
    for name, sup in sups.items():
        if bool((sup.count < 0).any()):
            raise RuntimeError(f"{name}: a warped row has more than {SUPPORT_CAP} tokens; "
                               "use the dense warped entry points for such rows")
    return sups


def build_profile(batch, n_s=10, n_a=10, n_x=10, warp=None):
    """Profile table and information figures from one batch of logits (GPU)."""
    z_t, z_d, z_c, x = batch["z_t"], batch["z_d"], batch["z_c"], batch["x"]
    B, k, V = z_d.shape
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    lse_d, lse_c, S, A, ratio = (f32(B, k) for _ in range(5))
    ws = alloc_workspace(B, k, V, B_._dtype_tag(z_d))
    edges_s = torch.linspace(0, 1, n_s + 1, device="cuda", dtype=torch.float32)
    edges_a = torch.linspace(0, 1, n_a + 1, device="cuda", dtype=torch.float32)
    counts = torch.zeros((n_s, n_a, n_x), dtype=torch.int32, device="cuda")
    sum_x = torch.zeros((n_s, n_a), dtype=torch.float64, device="cuda")
    table, info = f32(n_s, n_a), torch.zeros(3, dtype=torch.float64, device="cuda")
    if warp is None:
        sv_row_stats(z_d, z_c, x, lse_d, lse_c, S, A, None, None, ws)
        sv_accept_ratio(z_t, z_d, x, ratio, None, ws)
    else:
        sups = _compact(batch, warp)
        sv_row_stats_sparse(sups["z_d"], sups["z_c"], x, V, lse_d, lse_c, S, A)
        sv_accept_ratio_sparse(sups["z_t"], sups["z_d"], x, V, ratio)
    sv_profile_accumulate(S, A, ratio, edges_s, edges_a, n_x, counts, sum_x)
    sv_profile_finalize(counts, sum_x, table, info)
    torch.cuda.synchronize()
    return edges_s, edges_a, table, info.cpu().numpy()


def simulate(make_batch, latency, steps, profile, warp=None):
    """Run `steps` decode steps on fresh batches; returns SD and SV totals."""
    edges_s, edges_a, table, _ = profile
    first = make_batch(0)
    B, k, V = first["z_d"].shape
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    lse_d, lse_c, S, A, p_hat = (f32(B, k) for _ in range(5))
    gamma, offs, total = i32(B), i32(B + 1), i32(1)
    tokens, n_acc, flags = i32(B, k + 1), i32(B), i32(B)
    ws = alloc_workspace(B, k, V, B_._dtype_tag(first["z_d"]))
    lat = torch.as_tensor(latency, dtype=torch.float32).cuda()
    res = {m: dict(accepted=0, verified=0, latency=0.0) for m in ("sd", "sv")}
    for t in range(steps):
        b = first if t == 0 else make_batch(t)
        z_t, z_d, z_c, x = b["z_t"], b["z_d"], b["z_c"], b["x"]
        sups = None if warp is None else _compact(b, warp)
        # plain speculative decoding: verify everything
        if warp is None:
            sv_verify_sample(z_t, None, z_d, x, None, 1234, t, tokens, n_acc, flags, None, ws)
        else:
            sv_verify_sample_sparse(sups["z_t"], None, sups["z_d"], x, None, V, 1234, t, tokens, n_acc, flags)
        torch.cuda.synchronize()
        res["sd"]["accepted"] += int(n_acc.sum())
        res["sd"]["verified"] += B * k
        res["sd"]["latency"] += float(latency[B * k])
        # speculative verification: verify what the estimate says is worth it
        if warp is None:
            sv_row_stats(z_d, z_c, x, lse_d, lse_c, S, A, None, None, ws)
        else:
            sv_row_stats_sparse(sups["z_d"], sups["z_c"], x, V, lse_d, lse_c, S, A)
        sv_accept_estimate(S, A, edges_s, edges_a, table, p_hat, None)
        sv_select_length(p_hat, lat, SV_BATCH_GREEDY, gamma, offs, total)
        if warp is None:
            sv_verify_sample(z_t, None, z_d, x, gamma, 1234, t, tokens, n_acc, flags, None, ws)
        else:
            sv_verify_sample_sparse(sups["z_t"], None, sups["z_d"], x, gamma, V, 1234, t, tokens, n_acc, flags)
        torch.cuda.synchronize()
        M = int(total.item())
        res["sv"]["accepted"] += int(n_acc.sum())
        res["sv"]["verified"] += M
        res["sv"]["latency"] += float(latency[M])
    for m in res:
        r = res[m]
        r["goodput"] = r["accepted"] / r["latency"] if r["latency"] else 0.0
        r["accept_rate"] = r["accepted"] / r["verified"] if r["verified"] else 0.0
        r["mean_verified_per_seq"] = r["verified"] / (steps * B)
    return res


def main():
    import svgen
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--B", type=int, default=None)
    ap.add_argument("--V", type=int, default=None)
    ap.add_argument("--t0", type=float, default=30.0)
    ap.add_argument("--d", type=float, default=0.08)
    ap.add_argument("--m0", type=int, default=128)
    ap.add_argument("--temperature", type=float, default=None)
    ap.add_argument("--top-k", type=int, default=0)
    ap.add_argument("--top-p", type=float, default=1.0)
    args = ap.parse_args()
    warp = None if args.temperature is None else (float(np.float32(args.temperature)), args.top_k, args.top_p)

    def mk(seed):
        b = svgen.make_config(args.config, seed=seed, B=args.B, V=args.V, device="cuda")
        if warp is not None:                       # drafted tokens come from the warped draft distribution
            sup = Supports(b["z_d"].shape[0] * b["z_d"].shape[1], SUPPORT_CAP)
            sv_warp_compact(b["z_d"], warp[0], warp[1], warp[2], sup)
            g = torch.Generator(device="cuda")
            g.manual_seed(seed)
            listed = torch.arange(SUPPORT_CAP, device="cuda")[None, :] < sup.count[:, None]
            pick = torch.multinomial(torch.where(listed, sup.prob, torch.zeros_like(sup.prob)).float(), 1,
                                     generator=g)
            b["x"] = sup.token.gather(1, pick).reshape(b["x"].shape).to(torch.int32).contiguous()
        return b
    held = mk(777_000)
    Bn, k = held["B"], held["k"]
    latency = svgen.latency_table(Bn * k, t0=args.t0, d=args.d, m0=args.m0)
    profile = build_profile(held, warp=warp)
    res = simulate(lambda t: mk(888_000 + t), latency, args.steps, profile, warp=warp)
    out = {"workload": held["name"], "B": Bn, "k": k, "V": held["V"], "steps": args.steps,
           "warp": None if warp is None else {"temperature": warp[0], "top_k": warp[1], "top_p": warp[2]},
           "profile_info_bits": {"H_X": float(profile[3][0]), "H_X_given_SA": float(profile[3][1]),
                                 "info_gain": float(profile[3][2])},
           "sd": res["sd"], "sv": res["sv"],
           "sv_over_sd_goodput": res["sv"]["goodput"] / res["sd"]["goodput"] if res["sd"]["goodput"] else None}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
