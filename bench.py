#!/usr/bin/env python3
"""Benchmark of the SV decode-step hot path on one MI355X.

A step = the four C-ABI calls chained on one stream over one batch of synthetic
logits resident in HBM:
    sv_row_stats -> sv_accept_estimate -> sv_select_length -> sv_verify_sample
Default workload: the headline configuration B=64, k=8, V=152064, bf16, with
verification at full length (gamma = k for every sequence), which is the 1088-row
workload the metric is quoted on; the selected lengths are still computed every
step.  `--config 4` (B=64, k=16) runs the ragged chain instead: the lengths come
from sv_select_length on the device, the target rows are packed for exactly those
lengths (outside the timed region) and verification reads only them.  Inputs
rotate over several distinct copies so that no step finds its logits in the
256 MB Infinity Cache.

Prints one JSON line: whole-step throughput in logit rows/s; the HBM roofline of
the dominant kernel from hipEvents recorded around every launch of it (traffic
from the committed rocprofv3 counter summary of the same workload, if there is
one); the same for the other kernels and for the sv_verify_sample call as a
whole; the CPU oracle timed on this machine on one core and on all of them; and a
short timing of the other configurations.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import tempfile
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0        # MI355X published HBM3E bandwidth
CDF_ABS_BAND = 1e-6          # resolution of the HIP path's fp32 sampling weights (comparison band)
METRIC = "SV verify step: logit rows/s + achieved HBM GB/s (B=64, k=8, V=152064 bf16)"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, help="0-based index into svgen.CONFIGS")
    ap.add_argument("--copies", type=int, default=4, help="distinct input copies rotated over")
    ap.add_argument("--dense", action="store_true", help="config 4: verify all k tokens from dense target rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="CPU work per oracle leg (1 core, N cores)")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay timing")
    ap.add_argument("--no-other-configs", action="store_true", help="skip the short timing of the other configs")
    ap.add_argument("--no-profile-pass", action="store_true",
                    help="skip the timing of the profile-construction pass")
    ap.add_argument("--no-warped", action="store_true",
                    help="skip the timing of the step on temperature/top-k/top-p warped distributions")
    ap.add_argument("--verify", choices=("plain", "chained"), default="plain",
                    help="chained: the whole run uses sv_verify_sample_chained (draft normalisers from "
                         "sv_row_stats; rows counted = rows swept); default: the four independent calls")
    ap.add_argument("--no-chained", action="store_true",
                    help="skip the timing of the step with sv_verify_sample_chained")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for rocprofv3 byte counters)")
    return ap.parse_args()


class Hip:
    """The few HIP runtime calls the bench needs for its own events."""

    def __init__(self):
        self.lib = ctypes.CDLL("libamdhip64.so")
        self.lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.lib.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]

    def event(self):
        e = ctypes.c_void_p()
        rc = self.lib.hipEventCreate(ctypes.byref(e))
        assert rc == 0, f"hipEventCreate -> {rc}"
        return e

    def record(self, e, stream_handle):
        rc = self.lib.hipEventRecord(e, ctypes.c_void_p(stream_handle))
        assert rc == 0, f"hipEventRecord -> {rc}"

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.lib.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, f"hipEventElapsedTime -> {rc}"
        return ms.value

    def elapsed_ms_or_none(self, a, b):
        """None when the events were never recorded (a kernel the call did not launch)."""
        ms = ctypes.c_float()
        if self.lib.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0:
            return ms.value
        self.lib.hipGetLastError()          # the failed query must not be taken for a failed launch later
        return None

    def destroy(self, *events):
        for e in events:
            self.lib.hipEventDestroy(e)


def read_traffic(workload, kernel):
    """Measured HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of
    this workload (profiles/hbm_traffic_<workload>.txt), or None when there is none."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith(f"traffic_bytes_per_launch[{kernel}]"):
            return float(line.split("=")[1].split()[0])
    return None


# ---------------------------------------------------------------------------------- CPU legs
def cpu_legs(args, cfgdesc, cpu_cfg, ragged, tables):
    """The oracle as it stands on the canonical batch, before anything touches the GPU:
    one process, then one worker per core (sequences split among them).  Returns the
    oracle's results for the parity check and the two baselines."""
    import numpy as np
    import svgen
    from oracle import parallel as OP
    from oracle import sv_oracle as O

    edges_s, edges_a, table, lat = tables
    B, k, V = cfgdesc["B"], cfgdesc["k"], cfgdesc["V"]
    eb = 2 if cfgdesc["dtype"] == "bf16" else 4
    zt, zd, zc = (svgen.to_numpy_bits(cpu_cfg[n]) for n in ("z_t", "z_d", "z_c"))
    x = cpu_cfg["x"].numpy()

    def one_core():
        r = O.row_stats(zd, zc, x)
        p, _ = O.accept_estimate(r["S"].astype(np.float32), r["A"].astype(np.float32), edges_s, edges_a, table)
        g, offs, _ = O.select_length(p, lat)
        if ragged:
            packed = np.concatenate([zt[b, :g[b] + 1] for b in range(B)], axis=0)
            v = O.verify_sample(packed, zd, x, gamma=g, t_offsets=offs, seed=0, step=0, cdf_abs_band=CDF_ABS_BAND)
        else:
            v = O.verify_sample(zt, zd, x, seed=0, step=0, cdf_abs_band=CDF_ABS_BAND)
        return dict(S=r["S"], A=r["A"], p_hat=p, gamma=g, t_offsets=offs, tokens=v["tokens"],
                    n_accept=v["n_accept"], flags=v["flags"])

    reps, c0 = 0, time.perf_counter()
    while True:
        ref = one_core()
        reps += 1
        c1 = time.perf_counter()
        if c1 - c0 >= args.cpu_seconds or reps >= 50:
            break
    g = ref["gamma"]
    verify_rows = int(np.sum(2 * g + 1)) if ragged else B * (2 * k + 1)
    rows = 2 * B * k + verify_rows
    cpu_s = (c1 - c0) / reps
    what = ("the whole canonical batch: %d sequences, %d logit rows, all four calls%s"
            % (B, rows, ", verification of the selected lengths on packed target rows" if ragged else ""))
    baseline = {"value": round(rows / cpu_s, 2), "unit": "rows/s", "cores": 1, "kind": "oracle",
                "sample": f"{what}, repeated {reps}x = {c1 - c0:.1f} s of CPU work",
                "GBps": round(rows * V * eb / cpu_s * 1e-9, 4)}

    # N cores: the same step, sequences split over one worker process per core
    n = max(1, min(len(os.sched_getaffinity(0)), 16, B))
    base = "/dev/shm" if os.path.isdir("/dev/shm") else None
    d = tempfile.mkdtemp(prefix="svbench_", dir=base)
    pool = OP.make_pool(n)
    try:
        zt_par = np.concatenate([zt[b, :g[b] + 1] for b in range(B)], axis=0) if ragged else zt
        OP.save_inputs(d, zt_par, zd, zc, x)
        reps_n, n0 = 0, time.perf_counter()
        while True:
            par = OP.step(pool, n, d, B, edges_s, edges_a, table, lat, seed=0, step_index=0,
                          verify_selected=ragged, packed=ragged, cdf_abs_band=CDF_ABS_BAND)
            reps_n += 1
            n1 = time.perf_counter()
            if n1 - n0 >= args.cpu_seconds or reps_n >= 200:
                break
    finally:
        pool.close()
        pool.join()
        OP.remove_inputs(d)
    for name in ("p_hat", "gamma", "tokens", "n_accept", "flags"):
        assert np.array_equal(par[name], ref[name]), f"N-core oracle differs from the 1-core oracle in {name}"
    par_s = (n1 - n0) / reps_n
    baseline["n_core"] = {"value": round(rows / par_s, 2), "unit": "rows/s", "cores": n, "kind": "oracle",
                          "sample": f"the same batch split by sequence over {n} worker processes "
                                    f"(multiprocessing, spawn), repeated {reps_n}x = {n1 - n0:.1f} s of wall time",
                          "GBps": round(rows * V * eb / par_s * 1e-9, 4)}
    return ref, baseline


# ---------------------------------------------------------------------------------- GPU step
class Runner:
    """Device buffers of one configuration and its decode step."""

    def __init__(self, P, svgen, torch, idx, n_copies, cpu_cfg=None, ragged=False):
        self.P, self.torch = P, torch
        self.desc = svgen.CONFIGS[idx]
        self.B, self.k, self.V = self.desc["B"], self.desc["k"], self.desc["V"]
        self.eb = 2 if self.desc["dtype"] == "bf16" else 4
        self.tag = P.SV_BF16 if self.eb == 2 else P.SV_F32
        self.ragged = ragged
        self.chained = False     # True: the three-call form (sv_estimate_select, sv_verify_sample_chained)
        B, k, V = self.B, self.k, self.V
        self.copies = []
        if cpu_cfg is not None:      # copy 0 = the canonical CPU-seeded batch (the one the oracle gets)
            self.copies.append({n: cpu_cfg[n].cuda() for n in ("z_t", "z_d", "z_c", "x")})
        r = 1
        while len(self.copies) < n_copies:       # the others are drawn on the GPU with the same recipe
            c = svgen.make_config(idx, seed=1000 + idx + 100 * r, device="cuda")
            self.copies.append({n: c[n] for n in ("z_t", "z_d", "z_c", "x")})
            r += 1
        edges_s, edges_a, table = svgen.profile_table(10, 10)
        cu = lambda a: torch.as_tensor(a).cuda()
        self.d_es, self.d_ea, self.d_tab = cu(edges_s), cu(edges_a), cu(table)
        self.d_lat = cu(svgen.latency_table(B * k))
        f32 = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
        i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
        self.lse_d, self.lse_c, self.S, self.A, self.p_hat = (f32(B, k) for _ in range(5))
        self.gamma, self.offs, self.total = i32(B), i32(B + 1), i32(1)
        self.tokens, self.n_acc, self.flags = i32(B, k + 1), i32(B), i32(B)
        self.ws = P.alloc_workspace(B, k, V, self.tag)
        self.stream = torch.cuda.current_stream()
        self.row_bytes = V * self.eb
        self.stats_rows = 2 * B * k
        self.verify_rows = [B * (2 * k + 1)] * len(self.copies)
        if ragged:
            # lengths of every copy from the chain itself, target rows packed for exactly those
            # lengths: what the target model's forward would hand over.  Not timed.
            self.verify_rows = []
            for c in self.copies:
                self.select(c)
                torch.cuda.synchronize()
                g = self.gamma.cpu()
                idx_rows = torch.cat([b * (k + 1) + torch.arange(int(g[b]) + 1) for b in range(B)]).cuda()
                c["z_t_packed"] = c["z_t"].reshape(B * (k + 1), V)[idx_rows].contiguous()
                self.verify_rows.append(int((2 * g + 1).sum()))
                del c["z_t"]
            torch.cuda.empty_cache()

    def select(self, c, s=None):
        P, s = self.P, (s or self.stream)
        P.sv_row_stats(c["z_d"], c["z_c"], c["x"], self.lse_d, self.lse_c, self.S, self.A, None, None, self.ws, s)
        if self.chained:     # the serving form of the step: estimate and selection in one launch as well
            P.sv_estimate_select(self.S, self.A, self.d_es, self.d_ea, self.d_tab, self.d_lat, P.SV_BATCH_GREEDY,
                                 self.p_hat, self.gamma, self.offs, self.total, None, s)
            return
        P.sv_accept_estimate(self.S, self.A, self.d_es, self.d_ea, self.d_tab, self.p_hat, None, s)
        P.sv_select_length(self.p_hat, self.d_lat, P.SV_BATCH_GREEDY, self.gamma, self.offs, self.total, s)

    def verify(self, c, seed, step, s=None):
        P, s = self.P, (s or self.stream)
        call = P.sv_verify_sample_chained if self.chained else P.sv_verify_sample
        if self.ragged:      # lengths and offsets as the selection left them on the device
            call(c["z_t_packed"], self.offs, c["z_d"], c["x"], self.gamma, seed, step,
                 self.tokens, self.n_acc, self.flags, None, self.ws, s)
        else:
            call(c["z_t"], None, c["z_d"], c["x"], None, seed, step,
                 self.tokens, self.n_acc, self.flags, None, self.ws, s)

    def step(self, i, seed=0, s=None):
        c = self.copies[i % len(self.copies)]
        self.select(c, s)
        self.verify(c, seed, i, s)

    def rows_per_step(self):
        return self.stats_rows + sum(self.verify_rows) / len(self.verify_rows)

    def settle_clocks(self, seconds=0.05):
        """Untimed steps before the warm-up: a GPU that has idled takes some tens of milliseconds of
        load to reach the clocks it then holds (a 20-step run straight after the set-up measured
        0.182-0.184 ms per step, the same 20 steps after this 0.171-0.172, a 200-step run 0.171)."""
        torch = self.torch
        t0 = time.perf_counter()
        i = 0
        while time.perf_counter() - t0 < seconds:
            for _ in range(16):
                self.step(i)
                i += 1
            torch.cuda.synchronize()

    def time_steps(self, warmup, steps):
        torch = self.torch
        step = self.step
        self.settle_clocks()
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def time_graphs(self, warmup, steps):
        """The same steps replayed from HIP graphs (one captured step per input copy)."""
        torch = self.torch
        step = self.step
        graphs = []
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for r in range(len(self.copies)):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(r, s=torch.cuda.current_stream())
                graphs.append(g)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        for i in range(warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for i in range(steps):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        return (time.perf_counter() - g0) * 1e3 / steps

    def time_kernels(self, hip, Bd, steps):
        """The same steps again with hipEvents around every kernel launch and around the whole
        sv_verify_sample call.  Returns ({kernel: samples_us}, verify_call_samples_us)."""
        import numpy as np
        names = {Bd.SV_KERNEL_ROW_STATS: "row_stats_stash_kernel", Bd.SV_KERNEL_ACCEPT_ESTIMATE: "accept_estimate_kernel",
                 Bd.SV_KERNEL_SELECT_LENGTH: "select_batch_kernel", Bd.SV_KERNEL_VERIFY_ROWS: "verify_rows_kernel",
                 Bd.SV_KERNEL_VERIFY_MASS: "verify_mass_kernel", Bd.SV_KERNEL_VERIFY_PICK: "verify_pick_kernel"}
        P = self.P
        ev = {kid: [(hip.event(), hip.event()) for _ in range(steps)] for kid in names}
        for i in range(steps):
            for kid in names:
                P.sv_set_timing_events(kid, ev[kid][i][0], ev[kid][i][1])
            self.step(i)
        for kid in names:
            P.sv_set_timing_events(kid, None, None)
        self.torch.cuda.synchronize()
        samples = {}
        for kid in names:        # small batches run sv_verify_sample as one kernel: the other two taps stay silent
            t = [hip.elapsed_ms_or_none(a, b) for a, b in ev[kid]]
            if all(v is not None for v in t):
                samples[names[kid]] = np.array(t) * 1e3
        for kid in names:
            for a, b in ev[kid]:
                hip.destroy(a, b)
        # once more with one pair of events around the whole sv_verify_sample call (no events
        # between its kernels: each costs the stream 2-3 us)
        call = [(hip.event(), hip.event()) for _ in range(steps)]
        h = self.stream.cuda_stream
        for i in range(steps):
            c = self.copies[i % len(self.copies)]
            self.select(c)
            hip.record(call[i][0], h)
            self.verify(c, 0, i)
            hip.record(call[i][1], h)
        self.torch.cuda.synchronize()
        call_us = np.array([hip.elapsed_ms(a, b) for a, b in call]) * 1e3
        for a, b in call:
            hip.destroy(a, b)
        return samples, call_us


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (--gpus {args.gpus} requested); "
              "no multi-GPU path exists, run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import __graft_entry__
    __graft_entry__.ensure_built()          # loads what is built; builds only if nothing is
    import svgen

    t_setup = time.time()
    cfgdesc = svgen.CONFIGS[args.config]
    B, k, V = cfgdesc["B"], cfgdesc["k"], cfgdesc["V"]
    ragged = (args.config == 4) and not args.dense
    workload = cfgdesc["name"] if ragged or args.config != 4 else cfgdesc["name"].replace("_ragged", "_dense")
    if args.verify == "chained":
        workload += "_chained"
    cpu_cfg = svgen.make_config(args.config)
    edges_s, edges_a, table = svgen.profile_table(10, 10)
    lat = svgen.latency_table(B * k)

    # ---- CPU oracle first: it starts worker processes, which is done before the GPU is touched
    ref = cpu_baseline = None
    if not args.no_cpu_baseline:
        ref, cpu_baseline = cpu_legs(args, cfgdesc, cpu_cfg, ragged, (edges_s, edges_a, table, lat))

    import paper_2509_24328_amd as P
    from paper_2509_24328_amd import binding as Bd
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    run = Runner(P, svgen, torch, args.config, args.copies, cpu_cfg=cpu_cfg, ragged=ragged)
    chained_run = args.verify == "chained"
    run.chained = chained_run
    if chained_run:        # rows of the verification call = the target rows it sweeps, sum_b (gamma_b + 1)
        run.verify_rows = [(v + B) // 2 for v in run.verify_rows]
    copies, stream, ws = run.copies, run.stream, run.ws
    lse_d, lse_c, S, A, p_hat = run.lse_d, run.lse_c, run.S, run.A, run.p_hat
    gamma, offs, total, tokens, n_acc, flags = run.gamma, run.offs, run.total, run.tokens, run.n_acc, run.flags
    d_es, d_ea, d_tab, d_lat = run.d_es, run.d_ea, run.d_tab, run.d_lat
    f32 = lambda *s: torch.zeros(s, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device="cuda")
    row_bytes = run.row_bytes

    # ---- timed region: W warm-up steps, then exactly K steps between syncs
    ms_per_step = run.time_steps(args.warmup, args.steps)
    graph_ms = None if args.no_graph else run.time_graphs(args.warmup, args.steps)

    # ---- per-kernel and per-call hipEvent brackets over the same K steps
    hip = Hip()
    samples, call_us = run.time_kernels(hip, Bd, args.steps)
    us = {n: float(np.mean(v)) for n, v in samples.items()}

    # ---- algorithmic bytes per launch (each needed input byte once)
    verify_rows = sum(run.verify_rows) / len(run.verify_rows)
    stats_rows = run.stats_rows
    alg = {n: 0 for n in us}
    alg["verify_rows_kernel"] = verify_rows * row_bytes
    alg["row_stats_stash_kernel"] = stats_rows * row_bytes
    kernels = {}
    for n, t_us in us.items():
        kernels[n] = {"avg_us": round(t_us, 2), "median_us": round(float(np.median(samples[n])), 2),
                      "min_us": round(float(np.min(samples[n])), 2)}
        if alg[n]:
            gbs = alg[n] / t_us * 1e-3
            kernels[n].update({"algorithmic_bytes": int(alg[n]), "achieved_GBps": round(gbs, 1),
                               "frac_of_peak": round(gbs / PEAK_HBM_GBS, 4),
                               "traffic": read_traffic(workload, n)})
    dominant = max((n for n in us if alg[n]), key=lambda n: us[n])
    dom_gbs = alg[dominant] / us[dominant] * 1e-3
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(dom_gbs, 1), "peak": PEAK_HBM_GBS,
                "unit": "GB/s", "frac": round(dom_gbs / PEAK_HBM_GBS, 4),
                "traffic": read_traffic(workload, dominant), "avg_us": round(us[dominant], 2),
                "algorithmic_bytes": int(alg[dominant])}
    # the sv_verify_sample call as a whole (its three kernels between one pair of events)
    call_mean = float(np.mean(call_us))
    call_gbs = alg["verify_rows_kernel"] / call_mean * 1e-3
    mk_gbs = alg["verify_rows_kernel"] / us["verify_rows_kernel"] * 1e-3
    verify_call = {"rows": round(verify_rows, 1), "us": round(call_mean, 2),
                   "median_us": round(float(np.median(call_us)), 2), "min_us": round(float(np.min(call_us)), 2),
                   "rows_per_s": round(verify_rows / call_mean * 1e6, 1),
                   "algorithmic_bytes": int(alg["verify_rows_kernel"]),
                   "achieved_GBps": round(call_gbs, 1), "frac_of_peak": round(call_gbs / PEAK_HBM_GBS, 4),
                   "sum_of_kernel_brackets_us": round(sum(us[n] for n in us if n.startswith("verify_")), 2),
                   "metric_kernel": "verify_rows_kernel", "metric_kernel_GBps": round(mk_gbs, 1),
                   "metric_kernel_frac_of_peak": round(mk_gbs / PEAK_HBM_GBS, 4)}
    roofline["verify_call"] = {"us": verify_call["us"], "achieved": verify_call["achieved_GBps"],
                               "frac": verify_call["frac_of_peak"]}

    # ---- correctness on the timed buffers (copy 0 = the batch the oracle was run on)
    run.step(0, seed=0)
    torch.cuda.synchronize()
    got = dict(S=S.cpu().numpy(), A=A.cpu().numpy(), p_hat=p_hat.cpu().numpy(), gamma=gamma.cpu().numpy(),
               t_offsets=offs.cpu().numpy(), tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
               flags=flags.cpu().numpy())
    parity = None
    if ref is not None:
        near_bits = 2 | 8      # near tie, near CDF edge
        near = ((ref["flags"] | got["flags"].astype(np.uint32)) & near_bits) != 0
        ok = ~near
        bad = int(np.sum(got["n_accept"][ok] != ref["n_accept"][ok]))
        bad += int(np.sum(np.any(got["tokens"][ok] != ref["tokens"][ok], axis=1)))
        s_err = float(np.max(np.abs(got["S"] - ref["S"]) / ref["S"]))
        a_err = float(np.max(np.abs(got["A"] - ref["A"]) / ref["A"]))
        parity = {"sequences_checked": int(B), "token_or_count_mismatches_off_flag": bad,
                  "flagged_near_tie_or_edge": int(near.sum()), "max_rel_err_S": s_err, "max_rel_err_A": a_err,
                  "p_hat_equal": bool(np.array_equal(got["p_hat"], ref["p_hat"])),
                  "gamma_equal": bool(np.array_equal(got["gamma"], ref["gamma"])),
                  "offsets_equal": bool(np.array_equal(got["t_offsets"], ref["t_offsets"]))}
        assert bad == 0 and s_err < 1e-5 and a_err < 1e-5 and parity["gamma_equal"], parity

    # ---- the same step in its three-call form: sv_estimate_select (lookup and selection in one
    # launch) and sv_verify_sample_chained (the draft rows' normalisers come from what sv_row_stats
    # left in the workspace, so verification sweeps the target rows only).  Reported beside the
    # headline, which keeps the four independent calls and their byte count.
    chained_step = None
    if not args.no_chained and not chained_run:
        run.chained = True
        ch_ms = run.time_steps(args.warmup, args.steps)
        ch_samples, ch_call = run.time_kernels(hip, Bd, args.steps)
        run.step(0, seed=0)
        torch.cuda.synchronize()
        run.chained = False
        ch = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(), flags=flags.cpu().numpy())
        soft = ((ch["flags"] | got["flags"]) & (2 | 8)) != 0
        same = bool(np.array_equal(ch["tokens"][~soft], got["tokens"][~soft]) and
                    np.array_equal(ch["n_accept"][~soft], got["n_accept"][~soft]) and
                    np.array_equal(ch["flags"][~soft], got["flags"][~soft]))
        assert same and not (ch["flags"] & 64).any(), "chained verification differs from the plain call"
        t_rows = (verify_rows + B) / 2                      # sum_b (gamma_b + 1) target rows
        rows_us = float(np.mean(ch_samples["verify_rows_kernel"]))
        call_ch = float(np.mean(ch_call))
        chained_step = {"calls": "row_stats+estimate_select+verify_sample_chained",
                        "ms_per_step": round(ch_ms, 5),
                        "rows_swept_per_step": round(stats_rows + t_rows, 1),
                        "verify_rows_swept": round(t_rows, 1),
                        "verify_call_us": round(call_ch, 2),
                        "verify_rows_kernel_us": round(rows_us, 2),
                        "verify_rows_kernel_GBps": round(t_rows * row_bytes / rows_us * 1e-3, 1),
                        "kernel_us": {n: round(float(np.mean(v)), 2) for n, v in ch_samples.items()},
                        "same_tokens_counts_flags_as_plain_off_near_flags": same}

    # ---- the other configurations, briefly (their full-size parity is in tests/)
    other = None
    if not args.no_other_configs:
        other = []
        for idx in range(len(svgen.CONFIGS)):
            if idx == args.config:
                continue
            r2 = Runner(P, svgen, torch, idx, 2 if idx == 4 else 4, ragged=(idx == 4))
            ms = r2.time_steps(5, 40)
            gms = None if args.no_graph else r2.time_graphs(5, 40)
            smp, cus = r2.time_kernels(hip, Bd, 40)
            r2.chained = True
            ms3 = r2.time_steps(5, 40)
            r2.chained = False
            vr = sum(r2.verify_rows) / len(r2.verify_rows)
            other.append({"workload": r2.desc["name"], "ms_per_step": round(ms, 5),
                          "graph_replay_ms_per_step": None if gms is None else round(gms, 5),
                          "three_call_ms_per_step": round(ms3, 5),
                          "rows_per_step": round(r2.rows_per_step(), 1),
                          "rows_per_s": round(r2.rows_per_step() / (ms * 1e-3), 1),
                          "verify_rows": round(vr, 1), "verify_call_us": round(float(np.mean(cus)), 2),
                          "verify_call_GBps": round(vr * r2.row_bytes / float(np.mean(cus)) * 1e-3, 1),
                          "kernel_us": {n: round(float(np.mean(v)), 2) for n, v in smp.items()}})
            del r2
            torch.cuda.empty_cache()

    # ---- sv_row_stats with the optional outputs (KL, draft entropy, P_d(x): the signals of
    # the baseline predictors), same rotation of inputs; bracketed by the same timing tap
    kl_out, ent_out, pdx_out = f32(B, k), f32(B, k), f32(B, k)
    for i in range(3):
        c = copies[i % len(copies)]
        P.sv_row_stats(c["z_d"], c["z_c"], c["x"], lse_d, lse_c, S, A, kl_out, None, ws, stream,
                       entropy_d=ent_out, pd_x=pdx_out)
    torch.cuda.synchronize()
    xe = [(hip.event(), hip.event()) for _ in range(40)]
    for i, (e0, e1) in enumerate(xe):
        c = copies[i % len(copies)]
        P.sv_set_timing_events(Bd.SV_KERNEL_ROW_STATS, e0, e1)
        P.sv_row_stats(c["z_d"], c["z_c"], c["x"], lse_d, lse_c, S, A, kl_out, None, ws, stream,
                       entropy_d=ent_out, pd_x=pdx_out)
    P.sv_set_timing_events(Bd.SV_KERNEL_ROW_STATS, None, None)
    torch.cuda.synchronize()
    ext_us = float(np.mean([hip.elapsed_ms(a, b) for a, b in xe]) * 1e3)
    row_stats_extended = {"outputs": "S, A, KL, H(P_d), P_d(x)", "avg_us": round(ext_us, 2),
                          "achieved_GBps": round(alg["row_stats_stash_kernel"] / ext_us * 1e-3, 1)}

    # ---- profile-construction pass (the offline step before the hot path), timed
    # on a held-out batch of the same recipe: S, A from sv_row_stats, X from
    # sv_accept_ratio, 10x10 uniform grid, histogram, table + information gain
    profile_pass = None
    if not args.no_profile_pass:
        held = svgen.make_config(args.config, seed=5000 + args.config, device="cuda")
        ratio = f32(B, k)
        n_s = n_a = 10
        n_x = 10
        counts = torch.zeros((n_s, n_a, n_x), dtype=torch.int32, device="cuda")
        sum_x = torch.zeros((n_s, n_a), dtype=torch.float64, device="cuda")
        ptable = f32(n_s, n_a)
        info = torch.zeros(3, dtype=torch.float64, device="cuda")

        def profile_once():
            P.sv_row_stats(held["z_d"], held["z_c"], held["x"], lse_d, lse_c, S, A, None, None, ws, stream)
            P.sv_accept_ratio(held["z_t"], held["z_d"], held["x"], ratio, None, ws, stream)
            counts.zero_()
            sum_x.zero_()
            P.sv_profile_accumulate(S, A, ratio, d_es, d_ea, n_x, counts, sum_x, stream)
            P.sv_profile_finalize(counts, sum_x, ptable, info, stream)

        for _ in range(3):
            profile_once()
        torch.cuda.synchronize()
        reps = 20
        pe = [(hip.event(), hip.event()) for _ in range(reps)]
        p0 = time.perf_counter()
        for i in range(reps):
            P.sv_set_timing_events(Bd.SV_KERNEL_VERIFY_ROWS, pe[i][0], pe[i][1])
            profile_once()
        P.sv_set_timing_events(Bd.SV_KERNEL_VERIFY_ROWS, None, None)
        torch.cuda.synchronize()
        p1 = time.perf_counter()
        ratio_rows_us = float(np.mean([hip.elapsed_ms(a, b) for a, b in pe]) * 1e3)
        ratio_bytes = 2 * B * k * row_bytes
        hinfo = info.cpu().numpy()
        profile_pass = {"samples": B * k, "grid": f"{n_s}x{n_a} uniform, {n_x} X bins",
                        "ms_per_pass": round((p1 - p0) * 1e3 / reps, 4),
                        "accept_ratio_rows_kernel_us": round(ratio_rows_us, 2),
                        "accept_ratio_rows_kernel_GBps": round(ratio_bytes / ratio_rows_us * 1e-3, 1),
                        "H_X_bits": round(float(hinfo[0]), 4), "H_X_given_SA_bits": round(float(hinfo[1]), 4),
                        "info_gain_bits": round(float(hinfo[2]), 4)}
        if not args.no_cpu_baseline:
            from oracle import profile_oracle as PO
            from oracle import sv_oracle as O
            nq = min(B, 8)                       # a slice keeps the oracle leg short
            hz = {n: svgen.to_numpy_bits(held[n][:nq]) for n in ("z_t", "z_d", "z_c")}
            hx = held["x"][:nq].cpu().numpy()
            rs_ = O.row_stats(hz["z_d"], hz["z_c"], hx)
            rr_, _ = PO.accept_probability_ratio(hz["z_t"], hz["z_d"], hx)
            P.sv_row_stats(held["z_d"], held["z_c"], held["x"], lse_d, lse_c, S, A, None, None, ws, stream)
            torch.cuda.synchronize()
            got_ratio = ratio.cpu().numpy()[:nq]
            rel = float(np.max(np.abs(got_ratio - rr_) / np.abs(rr_)))
            relS = float(np.max(np.abs(S.cpu().numpy()[:nq] - rs_["S"]) / rs_["S"]))
            profile_pass["parity"] = {"sequences_checked": nq, "max_rel_err_ratio": rel, "max_rel_err_S": relS}
            assert rel < 1e-5 and relS < 1e-5, profile_pass
        del held

    # ---- the same step on warped distributions (temperature 0.7, top-k 20, top-p 0.8
    # for all three models: one row of the paper's table of sampling hyper-parameters):
    # three cutoff passes, then the warped indicators and the warped verification
    warped_step = None
    if not args.no_warped:
        wT, wK, wP = float(np.float32(0.7)), 20, 0.8
        c0 = copies[0]
        if "z_t" not in c0:                   # ragged run: the dense target rows of copy 0 again
            c0 = dict(c0, z_t=cpu_cfg["z_t"].cuda())
        cut_t, cut_d, cut_c = f32(B * (k + 1)), f32(B * k), f32(B * k)

        w_zs, w_cuts = [c0["z_t"], c0["z_d"], c0["z_c"]], [cut_t, cut_d, cut_c]

        def warped_once(i):
            P.sv_warp_cutoffs_multi(w_zs, wT, wK, wP, w_cuts, None, stream)     # the three tensors in one launch
            P.sv_row_stats_warped(c0["z_d"], c0["z_c"], c0["x"], wT, cut_d, wT, cut_c, lse_d, lse_c, S, A,
                                  None, None, ws, stream)
            P.sv_accept_estimate(S, A, d_es, d_ea, d_tab, p_hat, None, stream)
            P.sv_select_length(p_hat, d_lat, P.SV_BATCH_GREEDY, gamma, offs, total, stream)
            P.sv_verify_sample_warped(c0["z_t"], None, c0["z_d"], c0["x"], None, wT, cut_t, wT, cut_d, 0, i,
                                      tokens, n_acc, flags, None, ws, stream)

        def warped_once3(i):        # three-call form: estimate + selection in one launch, chained verification
            P.sv_warp_cutoffs_multi(w_zs, wT, wK, wP, w_cuts, None, stream)
            P.sv_row_stats_warped(c0["z_d"], c0["z_c"], c0["x"], wT, cut_d, wT, cut_c, lse_d, lse_c, S, A,
                                  None, None, ws, stream)
            P.sv_estimate_select(S, A, d_es, d_ea, d_tab, d_lat, P.SV_BATCH_GREEDY, p_hat, gamma, offs, total, None, stream)
            P.sv_verify_sample_warped_chained(c0["z_t"], None, c0["z_d"], c0["x"], None, wT, cut_t, wT, cut_d, 0, i,
                                              tokens, n_acc, flags, None, ws, stream)

        reps = 20
        for i in range(3):
            warped_once3(i)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        for i in range(reps):
            warped_once3(i)
        torch.cuda.synchronize()
        warped3_ms = (time.perf_counter() - w0) * 1e3 / reps
        assert not (flags.cpu().numpy() & 64).any(), "chained warped verification did not find the statistics pass"
        tokens3, n_acc3 = tokens.clone(), n_acc.clone()
        for i in range(3):
            warped_once(i)
        torch.cuda.synchronize()
        w0 = time.perf_counter()
        for i in range(reps):
            warped_once(i)
        torch.cuda.synchronize()
        w1 = time.perf_counter()
        # (both forms ended on step reps - 1: same uniforms, so the same accept counts off the near flags)
        same3 = bool(np.array_equal(n_acc3.cpu().numpy()[(flags.cpu().numpy() & (2 | 8)) == 0],
                                    n_acc.cpu().numpy()[(flags.cpu().numpy() & (2 | 8)) == 0]))
        ce0, ce1 = hip.event(), hip.event()
        torch.cuda.synchronize()
        # the cutoff pass alone (all three tensors in one launch), bracketed by events on the launch
        # stream; then one launch per tensor for comparison
        cut_t_, cut3_t_ = [], []
        for _ in range(10):
            hip.record(ce0, stream.cuda_stream)
            P.sv_warp_cutoffs_multi(w_zs, wT, wK, wP, w_cuts, None, stream)
            hip.record(ce1, stream.cuda_stream)
            torch.cuda.synchronize()
            cut_t_.append(hip.elapsed_ms(ce0, ce1) * 1e3)
            hip.record(ce0, stream.cuda_stream)
            for z_, c_ in zip(w_zs, w_cuts):
                P.sv_warp_cutoffs(z_, wT, wK, wP, c_, None, stream)
            hip.record(ce1, stream.cuda_stream)
            torch.cuda.synchronize()
            cut3_t_.append(hip.elapsed_ms(ce0, ce1) * 1e3)
        cut_us, cut3_us = float(np.mean(cut_t_)), float(np.mean(cut3_t_))
        warped_step = {"temperature": 0.7, "top_k": wK, "top_p": wP,
                       "ms_per_step": round((w1 - w0) * 1e3 / reps, 4),
                       "three_call_ms_per_step": round(warped3_ms, 4),
                       "three_call_n_accept_equal_off_near_flags": same3,
                       "cutoff_pass_us": round(cut_us, 1),
                       "cutoff_rows": B * (3 * k + 1),
                       "cutoff_pass_GBps": round(B * (3 * k + 1) * row_bytes / cut_us * 1e-3, 1),
                       "cutoff_pass_one_launch_per_tensor_us": round(cut3_us, 1)}

        # the repetition penalty of the same table row (1.05), timed on scratch copies of the three
        # tensors (it rewrites logits in place): 512 context tokens per sequence plus the drafted prefix
        rp_hist = torch.randint(0, V, (B, 512), dtype=torch.int32, device="cuda")
        rp_z = [c0["z_t"].clone(), c0["z_d"].clone(), c0["z_c"].clone()]
        P.sv_repetition_penalty_multi(rp_z, rp_hist, 1.05, x=c0["x"], stream=stream)
        torch.cuda.synchronize()
        rp_reps = 20
        r0 = time.perf_counter()
        for _ in range(rp_reps):
            for z_ in rp_z:
                P.sv_repetition_penalty(z_, rp_hist, 1.05, x=c0["x"], stream=stream)
        torch.cuda.synchronize()
        r1 = time.perf_counter()
        for _ in range(rp_reps):
            P.sv_repetition_penalty_multi(rp_z, rp_hist, 1.05, x=c0["x"], stream=stream)
        torch.cuda.synchronize()
        warped_step["repetition_penalty"] = {"penalty": 1.05, "context_tokens": 512, "rows": B * (3 * k + 1),
                                             "three_calls_us": round((r1 - r0) * 1e6 / rp_reps, 1),
                                             "one_launch_us": round((time.perf_counter() - r1) * 1e6 / rp_reps, 1)}
        del rp_z

        # the same warped step on compacted supports: one compaction pass per tensor, then
        # every later stage works on the few kept tokens of each row
        cap = 64
        sup_t, sup_d, sup_c = P.Supports(B * (k + 1), cap), P.Supports(B * k, cap), P.Supports(B * k, cap)
        s_tokens, s_nacc, s_flags = i32(B, k + 1), i32(B), i32(B)
        s_S, s_A = f32(B, k), f32(B, k)

        def sparse_once(i):
            P.sv_warp_compact_multi(w_zs, wT, wK, wP, [sup_t, sup_d, sup_c], None, None, stream)
            P.sv_row_stats_sparse(sup_d, sup_c, c0["x"], V, lse_d, lse_c, s_S, s_A, None, None, stream)
            P.sv_estimate_select(s_S, s_A, d_es, d_ea, d_tab, d_lat, P.SV_BATCH_GREEDY, p_hat, gamma, offs, total,
                                 None, stream)
            P.sv_verify_sample_sparse(sup_t, None, sup_d, c0["x"], None, V, 0, i, s_tokens, s_nacc, s_flags,
                                      None, stream)

        for i in range(3):
            sparse_once(i)
        torch.cuda.synchronize()
        q0 = time.perf_counter()
        for i in range(reps):
            sparse_once(i)
        torch.cuda.synchronize()
        q1 = time.perf_counter()
        counts = torch.cat([sup_t.count, sup_d.count, sup_c.count]).cpu().numpy()
        # both paths on the same step index: identical accept counts and tokens
        warped_once(5)
        sparse_once(5)
        torch.cuda.synchronize()
        same_n = bool(torch.equal(n_acc, s_nacc))
        near = ((flags | s_flags) & (2 | 8)) != 0
        same_tok = bool(torch.equal(tokens[~near], s_tokens[~near]))
        warped_step["compacted"] = {"cap": cap, "ms_per_step": round((q1 - q0) * 1e3 / reps, 4),
                                    "rows_not_compact": int((counts < 0).sum()),
                                    "mean_support": round(float(counts[counts > 0].mean()), 2),
                                    "n_accept_equal_dense_warped": same_n,
                                    "tokens_equal_dense_warped_off_near_flags": same_tok}
        assert same_n and same_tok, warped_step
        if not args.no_cpu_baseline:
            from oracle import sv_oracle as O
            from oracle import warp_oracle as WO
            nq = min(B, 4)
            zt_n, zd_n, zc_n = (svgen.to_numpy_bits(c0[n][:nq]) for n in ("z_t", "z_d", "z_c"))
            xq = c0["x"][:nq].cpu().numpy()
            y_t, _, f_t = WO.warp_rows(zt_n, wT, wK, wP)
            y_d, _, f_d = WO.warp_rows(zd_n, wT, wK, wP)
            y_c, _, f_c = WO.warp_rows(zc_n, wT, wK, wP)
            warped_once(7)
            torch.cuda.synchronize()
            rs_ = O.row_stats(y_d, y_c, xq)
            rv_ = O.verify_sample(y_t, y_d, xq, seed=0, step=7, cdf_abs_band=CDF_ABS_BAND)
            near = (f_t.any(1) | f_d.any(1) | f_c.any(1)) | ((rv_["flags"] & O.FLAG_NEAR_TIE) != 0)
            okq = ~near
            # disjoint supports give S = 0 exactly on both sides
            relS = float(np.max(np.abs(S.cpu().numpy()[:nq] - rs_["S"]) / np.maximum(rs_["S"], 1e-30)))
            same = bool(np.array_equal(n_acc.cpu().numpy()[:nq][okq], rv_["n_accept"][okq]))
            warped_step["parity"] = {"sequences_checked": int(okq.sum()), "max_rel_err_S": relS,
                                     "n_accept_equal": same}
            assert relS < 1e-5 and same, warped_step

    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    rows_per_step = run.rows_per_step()
    calls = ("row_stats+estimate_select+verify_sample_chained(" if chained_run else
             "row_stats+accept_estimate+select_length+verify_sample(") + \
        ("gamma from select_length, packed target rows)" if ragged else "gamma=k)")
    out = {
        "metric": METRIC,
        "value": round(rows_per_step / (ms_per_step * 1e-3), 1),
        "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": workload, "B": B, "k": k, "V": V, "logit_dtype": cfgdesc["dtype"],
                   "calls": calls, "rows_per_step": round(rows_per_step, 1), "row_stats_rows": stats_rows,
                   "verify_rows": round(verify_rows, 1), "input_copies_rotated": len(copies)},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "verify_step": verify_call,
        "chained_step": chained_step,
        "kernels": kernels,
        "sum_kernel_us": round(sum(us.values()), 2),
        "graph_replay": None if graph_ms is None else {
            "ms_per_step": round(graph_ms, 5), "rows_per_s": round(rows_per_step / (graph_ms * 1e-3), 1)},
        "parity": parity,
        "other_configs": other,
        "row_stats_extended": row_stats_extended,
        "profile_pass": profile_pass,
        "warped_step": warped_step,
        "mean_gamma_selected": float(np.mean(got["gamma"])),
        "mean_accepted": float(np.mean(got["n_accept"])),
        "setup_s": round(time.time() - t_setup, 1),
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
