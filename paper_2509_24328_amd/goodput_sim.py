"""Step-level goodput simulation on synthetic logits, entirely through the C ABI:
plain speculative decoding against verification lengths chosen from three
acceptance estimators - SV's (S, A) pair and the two prior predictor families the
paper discusses (Sec. 2 "Predicting Speculation Accuracy": the entropy of the
draft distribution; the draft's probability of its own token).

What the paper measures end to end with real models (goodput = accepted tokens
per unit time, Sec. 5 and Sec. 7.2) is modelled here per decode step:

  * profiles: for every estimator the mean acceptance probability per cell of its
              signal (appendix definition of the observed P(T | S, A), applied to
              each signal alike) is built on a held-out batch (distinct seed) with
              the profile pass (sv_row_stats, sv_accept_ratio, sv_quantile_edges,
              sv_profile_accumulate, sv_profile_finalize); (S, A) uses a 10 x 10
              uniform grid, the entropy H(P_d) and P_d(x) 100 equal-count cells
              each (second axis: one bin), so all three have the same resolution;
  * SD step:  every sequence verifies all k drafted tokens;
  * other steps: sv_row_stats -> sv_accept_estimate (the estimator's signal and
              table) -> sv_select_length picks the lengths, only those positions
              are verified;
  * cost:     latency[M] of the caller's latency table, M = drafted tokens sent to
              the target in the step (the paper's profiled verification latency).

Goodput of a run = accepted drafted tokens / sum of step latencies; the accept
rate is accepted / verified.  Only the qualitative picture can be compared with
the paper (its numbers need its models and hardware): SV trades a little
acceptance volume for much less verification work where drafts are poor, and the
(S, A) signal carries more information about acceptance than the other two.

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
                      sv_accept_ratio_sparse, sv_profile_accumulate, sv_profile_finalize, sv_quantile_edges,
                      sv_row_stats, sv_row_stats_sparse, sv_select_length, sv_verify_sample,
                      sv_verify_sample_sparse, sv_warp_compact)

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


ESTIMATORS = ("sv", "entropy", "probability")


def _signals(batch, sups, ws):
    """S, A, H(P_d), P_d(x) of a batch ([B, k] float32 device tensors)."""
    z_d, z_c, x = batch["z_d"], batch["z_c"], batch["x"]
    B, k, V = z_d.shape
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    lse_d, lse_c, S, A, kl, H, pdx = (f32(B, k) for _ in range(7))
    if sups is None:
        sv_row_stats(z_d, z_c, x, lse_d, lse_c, S, A, kl, None, ws, entropy_d=H, pd_x=pdx)
    else:
        sv_row_stats_sparse(sups["z_d"], sups["z_c"], x, V, lse_d, lse_c, S, A, kl, entropy_d=H, pd_x=pdx)
    return dict(S=S, A=A, H_d=H, pd_x=pdx)


def _axes(name, sig):
    if name == "sv":
        return sig["S"], sig["A"]
    zero = torch.zeros_like(sig["S"])
    return (sig["H_d"] if name == "entropy" else sig["pd_x"]), zero


def build_profiles(batch, cells=100, n_x=10, warp=None, estimators=ESTIMATORS):
    """{estimator: (edges_1, edges_2, table, info)} from one held-out batch (GPU);
    info = (H(X), H(X | signal), information gain) in bits."""
    z_t, z_d, x = batch["z_t"], batch["z_d"], batch["x"]
    B, k, V = z_d.shape
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    ws = alloc_workspace(B, k, V, B_._dtype_tag(z_d))
    sups = None if warp is None else _compact(batch, warp)
    sig = _signals(batch, sups, ws)
    ratio = f32(B, k)
    if warp is None:
        sv_accept_ratio(z_t, z_d, x, ratio, None, ws)
    else:
        sv_accept_ratio_sparse(sups["z_t"], sups["z_d"], x, V, ratio)
    out = {}
    for name in estimators:
        a1, a2 = _axes(name, sig)
        if name == "sv":
            n = int(round(cells ** 0.5))
            e1 = torch.linspace(0, 1, n + 1, device="cuda", dtype=torch.float32)
            e2 = e1.clone()
        else:
            hi = float(np.float32(np.log(V))) if name == "entropy" else 1.0
            e1 = f32(cells + 1)
            sv_quantile_edges(a1, cells, 0.0, hi, e1)
            e2 = torch.tensor([0.0, 1.0], device="cuda", dtype=torch.float32)
        n1, n2 = e1.numel() - 1, e2.numel() - 1
        counts = torch.zeros((n1, n2, n_x), dtype=torch.int32, device="cuda")
        sum_x = torch.zeros((n1, n2), dtype=torch.float64, device="cuda")
        table, info = f32(n1, n2), torch.zeros(3, dtype=torch.float64, device="cuda")
        sv_profile_accumulate(a1, a2, ratio, e1, e2, n_x, counts, sum_x)
        sv_profile_finalize(counts, sum_x, table, info)
        torch.cuda.synchronize()
        out[name] = (e1, e2, table, info.cpu().numpy())
    return out


def build_profile(batch, n_s=10, n_a=10, n_x=10, warp=None):
    """The (S, A) profile alone: (edges_s, edges_a, table, info)."""
    assert n_s == n_a
    return build_profiles(batch, cells=n_s * n_a, n_x=n_x, warp=warp, estimators=("sv",))["sv"]


def simulate(make_batch, latency, steps, profiles, warp=None, keep_steps=False):
    """Run `steps` decode steps on fresh batches under plain SD ("sd") and under every
    estimator of `profiles` ({name: (edges_1, edges_2, table, ...)} with device tensors; a
    bare (edges_s, edges_a, table, ...) tuple means the (S, A) estimator alone).  The same
    Philox step serves all of them; only the verified lengths differ.  Returns the totals
    per name; with keep_steps also "steps": per step and name the lengths, the number of
    verified tokens, the accept counts and the flags (host arrays), and the signals."""
    if not isinstance(profiles, dict):
        profiles = {"sv": profiles}
    first = make_batch(0)
    B, k, V = first["z_d"].shape
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.empty(s, dtype=torch.int32, device="cuda")
    p_hat = f32(B, k)
    edge = torch.empty((B, k), dtype=torch.uint8, device="cuda")
    gamma, offs, total = i32(B), i32(B + 1), i32(1)
    tokens, n_acc, flags = i32(B, k + 1), i32(B), i32(B)
    ws = alloc_workspace(B, k, V, B_._dtype_tag(first["z_d"]))
    lat = torch.as_tensor(latency, dtype=torch.float32).cuda()
    names = ("sd",) + tuple(profiles)
    res = {m: dict(accepted=0, verified=0, latency=0.0) for m in names}
    log = []
    for t in range(steps):
        b = first if t == 0 else make_batch(t)
        z_t, z_d, x = b["z_t"], b["z_d"], b["x"]
        sups = None if warp is None else _compact(b, warp)
        sig = _signals(b, sups, ws)
        rec = {}
        for m in names:
            near_edge = False
            if m == "sd":                       # plain speculative decoding: verify everything
                g, M = None, B * k
            else:                               # verify what the estimate says is worth it
                e1, e2, table = profiles[m][:3]
                a1, a2 = _axes(m, sig)
                sv_accept_estimate(a1, a2, e1, e2, table, p_hat, edge)
                sv_select_length(p_hat, lat, SV_BATCH_GREEDY, gamma, offs, total)
                g = gamma
            if warp is None:
                sv_verify_sample(z_t, None, z_d, x, g, 1234, t, tokens, n_acc, flags, None, ws)
            else:
                sv_verify_sample_sparse(sups["z_t"], None, sups["z_d"], x, g, V, 1234, t, tokens, n_acc, flags)
            torch.cuda.synchronize()
            if m != "sd":
                M = int(total.item())
                near_edge = bool(edge.any())
            res[m]["accepted"] += int(n_acc.sum())
            res[m]["verified"] += M
            res[m]["latency"] += float(latency[M])
            if keep_steps:
                rec[m] = dict(gamma=(np.full(B, k, np.int32) if g is None else gamma.cpu().numpy().copy()), M=M,
                              n_accept=n_acc.cpu().numpy().copy(), flags=flags.cpu().numpy().astype(np.uint32),
                              near_edge=near_edge)
        if keep_steps:
            rec["signals"] = {n: v.cpu().numpy() for n, v in sig.items()}
            log.append(rec)
    for m in names:
        r = res[m]
        r["goodput"] = r["accepted"] / r["latency"] if r["latency"] else 0.0
        r["accept_rate"] = r["accepted"] / r["verified"] if r["verified"] else 0.0
        r["mean_verified_per_seq"] = r["verified"] / (steps * B)
    if keep_steps:
        res["steps"] = log
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
    profiles = build_profiles(held, warp=warp)
    res = simulate(lambda t: mk(888_000 + t), latency, args.steps, profiles, warp=warp)
    sd_goodput = res["sd"]["goodput"]
    out = {"workload": held["name"], "B": Bn, "k": k, "V": held["V"], "steps": args.steps,
           "warp": None if warp is None else {"temperature": warp[0], "top_k": warp[1], "top_p": warp[2]},
           "H_X_bits": float(profiles["sv"][3][0]),
           "info_gain_bits": {m: float(profiles[m][3][2]) for m in profiles},
           "runs": res,
           "goodput_over_sd": {m: (res[m]["goodput"] / sd_goodput if sd_goodput else None) for m in profiles}}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
