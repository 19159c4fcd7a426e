"""Randomised GPU parity sweep: many small seeded problems with mixed shapes,
dtypes, noise scales, verification lengths and Philox seeds, so that rare
near-tie / CDF-edge situations and odd shapes get exercised."""
import numpy as np
import pytest
import torch

import svgen
from oracle import sv_oracle as O

import harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("block", range(6))
def test_random_problems(block):
    rng = np.random.default_rng(9000 + block)
    n_tie = n_edge = n_seq = 0
    for case in range(10):
        idx = int(rng.integers(0, 4))
        B = int(rng.integers(1, 9))
        k = int(rng.integers(1, 10))
        V = int(rng.choice([int(rng.integers(2, 300)), int(rng.integers(300, 9000)),
                            8 * int(rng.integers(1000, 5000)), 8192 * int(rng.integers(1, 4)) + int(rng.integers(0, 9))]))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        seed = int(rng.integers(0, 2 ** 31))
        cfg = svgen.make_config(idx, B=B, k=k, V=V, dtype=dtype, seed=seed)
        d = {n: cfg[n].cuda() for n in ("z_t", "z_d", "z_c", "x")}
        oi = H.oracle_inputs(cfg)
        ref = O.row_stats(oi["z_d"], oi["z_c"], oi["x"])
        with_kl = bool(rng.random() < 0.5)
        H.assert_row_stats(H.gpu_row_stats(d["z_d"], d["z_c"], d["x"], with_kl), ref, with_kl)
        gamma = rng.integers(0, k + 1, size=B).astype(np.int32) if rng.random() < 0.6 else None
        pseed, step = int(rng.integers(0, 2 ** 62)), int(rng.integers(0, 2 ** 31))
        vref = H.oracle_verify(oi["z_t"], oi["z_d"], oi["x"], gamma=gamma, seed=pseed, step=step)
        vgot = H.gpu_verify(d["z_t"], d["z_d"], d["x"], gamma=gamma, seed=pseed, step=step)
        t, e = H.assert_verify(vgot, vref, k)
        n_tie, n_edge, n_seq = n_tie + t, n_edge + e, n_seq + B
        H.assert_verify(H.gpu_verify_chained(d["z_t"], d["z_d"], d["z_c"], d["x"], gamma=gamma, seed=pseed, step=step),
                        vref, k)
        p = rng.random((B, k)).astype(np.float32)
        lat = svgen.latency_table(B * k, t0=float(rng.uniform(0.1, 30)), d=float(rng.uniform(0.01, 1)),
                                  m0=int(rng.integers(1, B * k + 1)))
        for mode, l in ((O.MODE_BATCH_GREEDY, lat), (O.MODE_PER_SEQUENCE, lat[:k + 1])):
            rg, ro, rm = O.select_length(p, l, mode)
            gg, go, gm = H.gpu_select_length(p, l, mode)
            assert gm == rm and np.array_equal(gg, rg) and np.array_equal(go, ro)
    print(f"\n  block {block}: {n_seq} sequences, near-tie {n_tie}, near-cdf-edge {n_edge}", flush=True)


def _warped_case(rng, zs, dtype, par, with_kl=True):
    """One problem through the dense warped entry points (GPU cutoffs) and through the
    compacted ones, both against the oracle on warped rows.  zs: float32 arrays z_t, z_d,
    z_c holding exactly the stored values; par: (T, K, P) per tensor.  Drafted tokens are
    drawn from the warped draft distribution.  Pairs / sequences touching a near-tie top-p
    decision are skipped.  Returns (sequence checks, compacted pairs, near-ties)."""
    from oracle import warp_oracle as W
    P = H.sv()
    B, k, V = zs["d"].shape
    d = {n: H.dev(z, dtype) for n, z in zs.items()}
    y, cut, fl, gcut, gfl, sup = {}, {}, {}, {}, {}, {}
    for name in ("t", "d", "c"):
        T, K, Pp = par[name]
        with np.errstate(all="ignore"):
            y[name], cut[name], fl[name] = W.warp_rows(zs[name], T, K, Pp)
        rows = zs[name].shape[0] * zs[name].shape[1]
        gcut[name] = torch.empty(rows, dtype=torch.float32, device="cuda")
        gf = torch.empty(rows, dtype=torch.int32, device="cuda")
        sup[name] = P.Supports(rows, 128)
        P.sv_warp_compact(d[name], T, K, Pp, sup[name], gcut[name], gf)
        torch.cuda.synchronize()
        gfl[name] = gf.cpu().numpy().astype(np.uint32).reshape(fl[name].shape)
    tie = lambda n: ((fl[n] | gfl[n]) & O.FLAG_NEAR_TIE) != 0
    pair_tie = tie("d") | tie("c")
    seq_tie = tie("t").any(1) | tie("d").any(1)
    x = rng.integers(0, V, size=(B, k)).astype(np.int32)
    for b in range(B):
        for i in range(k):
            r = y["d"][b, i]
            if np.isfinite(r).any() and not np.isnan(r).any() and not np.isposinf(r).any():
                p = np.exp(r - r[np.isfinite(r)].max())
                p[~np.isfinite(r)] = 0.0
                if p.sum() > 0:
                    x[b, i] = rng.choice(V, p=p / p.sum())
    xg = H.dev(x, torch.int32)
    with np.errstate(all="ignore"):
        ref = O.row_stats(y["d"], y["c"], x)
    f32 = lambda *s: torch.full(s, -7.0, dtype=torch.float32, device="cuda")
    i32 = lambda *s: torch.full(s, -5, dtype=torch.int32, device="cuda")
    ws = P.alloc_workspace(B, k, V, P.binding._dtype_tag(d["d"]))
    keep = ~pair_tie
    pick = lambda dct, m: {n: np.asarray(v)[m] for n, v in dct.items() if v is not None}
    # dense warped indicators
    o = dict(lse_d=f32(B, k), lse_c=f32(B, k), S=f32(B, k), A=f32(B, k), KL=f32(B, k) if with_kl else None,
             H_d=f32(B, k) if with_kl else None, pd_x=f32(B, k), flags=i32(B, k))
    P.sv_row_stats_warped(d["d"], d["c"], xg, par["d"][0], gcut["d"], par["c"][0], gcut["c"], o["lse_d"],
                          o["lse_c"], o["S"], o["A"], o["KL"], o["flags"], ws, entropy_d=o["H_d"], pd_x=o["pd_x"])
    torch.cuda.synchronize()
    H.assert_row_stats(pick({n: None if t is None else t.cpu().numpy() for n, t in o.items()}, keep), pick(ref, keep), with_kl)
    # compacted indicators
    P.sv_row_stats_sparse(sup["d"], sup["c"], xg, V, o["lse_d"], o["lse_c"], o["S"], o["A"], o["KL"], o["flags"],
                          entropy_d=o["H_d"], pd_x=o["pd_x"])
    torch.cuda.synchronize()
    got = {n: None if t is None else t.cpu().numpy() for n, t in o.items()}
    ks = keep & ((got["flags"].astype(np.uint32) & 32) == 0)
    H.assert_row_stats(pick(got, ks), pick(ref, ks), with_kl)
    # verification, dense warped and compacted
    gamma = rng.integers(0, k + 1, size=B).astype(np.int32) if rng.random() < 0.6 else None
    gg = None if gamma is None else H.dev(gamma, torch.int32)
    pseed, step = int(rng.integers(0, 2 ** 62)), int(rng.integers(0, 2 ** 31))
    with np.errstate(all="ignore"):
        vref = H.oracle_verify(y["t"], y["d"], x, gamma=gamma, seed=pseed, step=step)
    sub = lambda dct, m: {n: ([v[i] for i in np.flatnonzero(m)] if isinstance(v, list) else np.asarray(v)[m])
                          for n, v in dct.items()}
    n_seq = n_tie = 0
    for mode in ("dense", "chained", "sparse"):
        tokens, n_acc, flags, ratio = i32(B, k + 1), i32(B), i32(B), f32(B, k)
        if mode == "dense":
            P.sv_verify_sample_warped(d["t"], None, d["d"], xg, gg, par["t"][0], gcut["t"], par["d"][0],
                                      gcut["d"], pseed, step, tokens, n_acc, flags, ratio, ws)
        elif mode == "chained":      # draft normalisers from the sv_row_stats_warped call above (same ws)
            P.sv_verify_sample_warped_chained(d["t"], None, d["d"], xg, gg, par["t"][0], gcut["t"], par["d"][0],
                                              gcut["d"], pseed, step, tokens, n_acc, flags, ratio, ws)
        else:
            P.sv_verify_sample_sparse(sup["t"], None, sup["d"], xg, gg, V, pseed, step, tokens, n_acc, flags, ratio)
        torch.cuda.synchronize()
        vgot = dict(tokens=tokens.cpu().numpy(), n_accept=n_acc.cpu().numpy(),
                    flags=flags.cpu().numpy().astype(np.uint32), ratio=ratio.cpu().numpy())
        assert mode != "chained" or not (vgot["flags"] & 64).any()     # the statistics pass was found
        m = ~seq_tie & ((vgot["flags"] & 32) == 0)
        t, _ = H.assert_verify(sub(vgot, m), sub(vref, m), k)
        n_tie += t
        n_seq += int(m.sum())
    return n_seq, int(ks.sum()), n_tie


@pytest.mark.parametrize("block", range(4))
def test_random_warped_problems(block):
    """Random shapes and sampling hyper-parameters on the configurations' input recipes."""
    rng = np.random.default_rng(7700 + block)
    n_seq = n_tie = n_sparse = 0
    for case in range(8):
        idx = int(rng.integers(0, 4))
        B = int(rng.integers(1, 6))
        k = int(rng.integers(1, 7))
        V = int(rng.choice([int(rng.integers(2, 300)), int(rng.integers(300, 9000)),
                            8 * int(rng.integers(1000, 5000)), 8192 * int(rng.integers(1, 4)) + int(rng.integers(0, 9))]))
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        cfg = svgen.make_config(idx, B=B, k=k, V=V, dtype=dtype, seed=int(rng.integers(0, 2 ** 31)))
        oi = H.oracle_inputs(cfg)
        par = {}
        for name in ("t", "d", "c"):
            T = float(np.float32(rng.choice([0.6, 0.7, 0.95, 1.0, 1.3])))
            K = int(rng.choice([0, 1, 5, 20, 50]))
            Pp = float(rng.choice([1.0, 0.9, 0.8, 0.6]))
            par[name] = (T, K, Pp)
        zs = {n: O.upcast(oi["z_" + n]).astype(np.float32) for n in ("t", "d", "c")}   # exactly the stored values
        s, p, t = _warped_case(rng, zs, cfg["z_d"].dtype, par)
        n_seq, n_sparse, n_tie = n_seq + s, n_sparse + p, n_tie + t
    print(f"\n  warped block {block}: {n_seq} sequence checks, {n_sparse} compacted pairs, near-tie {n_tie}", flush=True)
    assert n_seq >= 20 and n_sparse >= 20


def _adversarial_rows(rng, B, k, V, bf16):
    """Gaussian logits with, row by row, one of: a huge or tiny scale, a huge common
    offset, a mask (-inf or one of its finite stand-ins) over 10-99 % of the entries,
    integer values (ties), a constant row, a one-hot row."""
    z_t = (2 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    z_d = (z_t[:, :k] + rng.standard_normal((B, k, V)) * rng.choice([0.0, 0.3, 1.0, 3.0])).astype(np.float32)
    z_c = (z_t[:, :k] + rng.standard_normal((B, k, V)) * rng.choice([0.0, 0.3, 1.0, 3.0])).astype(np.float32)
    for z in (z_t, z_d, z_c):
        for row in z.reshape(-1, V):
            r = rng.random()
            if r < 0.15:
                row *= rng.choice([1e-3, 30.0, 1e3, 1e5])
            elif r < 0.30:
                row += rng.choice([-1e6, -1e4, -100.0, 100.0, 1e4, 1e6])
            elif r < 0.50:
                keep = rng.random(V) >= rng.choice([0.1, 0.5, 0.9, 0.99])
                keep[rng.integers(V)] = True
                row[~keep] = rng.choice([-np.inf, -1e30, float(np.finfo(np.float32).min), -1e9, -65504.0])
            elif r < 0.58:
                row[:] = np.round(row)
            elif r < 0.62:
                row[:] = row[0]
            elif r < 0.66:
                j = rng.integers(V)
                row[:] = -np.inf
                row[j] = rng.choice([0.0, 50.0, -50.0])
    x = rng.integers(0, V, size=(B, k)).astype(np.int32)
    if bf16:
        z_t, z_d, z_c = (torch.from_numpy(z).to(torch.bfloat16).float().numpy() for z in (z_t, z_d, z_c))
    return z_t, z_d, z_c, x


@pytest.mark.parametrize("block", range(4))
def test_random_adversarial_values(block):
    """sv_row_stats and sv_verify_sample against the oracle on rows far from the recipe of
    the configurations: logits of size 1e6, one-hot and constant rows, vocabularies of 1-17
    entries, masks written as -1e30 / the lowest finite number / -65504.  Drafted tokens
    are arbitrary, so tokens without mass under either model occur."""
    n_seq = n_tie = 0
    for case in range(40):
        rng = np.random.default_rng(31000 + 100 * block + case)
        bf16 = bool(case % 2)
        dtype = torch.bfloat16 if bf16 else torch.float32
        V = int(rng.choice([1, 2, 3, 7, 8, 17, 64, 300, 1000, 4096, 5001, 20000, 33000]))
        B, k = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        z_t, z_d, z_c, x = _adversarial_rows(rng, B, k, V, bf16)
        with np.errstate(all="ignore"):         # exp of +-1e6 inside the oracle's min(1, .) and ratios
            ref = O.row_stats(z_d, z_c, x)
            vref = H.oracle_verify(z_t, z_d, x, seed=case, step=block)
        # KL is left out: draft mass on a masked companion entry makes it about -mask
        got = H.gpu_row_stats(H.dev(z_d, dtype), H.dev(z_c, dtype), H.dev(x), with_kl=False)
        H.assert_row_stats(got, ref, with_kl=False)
        vgot = H.gpu_verify(H.dev(z_t, dtype), H.dev(z_d, dtype), H.dev(x), seed=case, step=block)
        t, _ = H.assert_verify(vgot, vref, k)
        n_seq, n_tie = n_seq + B, n_tie + t
        H.assert_verify(H.gpu_verify_chained(H.dev(z_t, dtype), H.dev(z_d, dtype), H.dev(z_c, dtype), H.dev(x),
                                             seed=case, step=block), vref, k)
    print(f"\n  block {block}: {n_seq} sequences, near-tie {n_tie}", flush=True)


@pytest.mark.parametrize("block", range(3))
def test_random_adversarial_values_warped(block):
    """The warped and compacted entry points on the adversarial rows above, with
    temperatures from 1e-3 to 1e3, top-k from 1 to V and top-p from 0.01 to 1.  Problems
    outside the documented range of the logits (|z| / T beyond 2^29 / log2 e for an entry
    that is no mask) are left out."""
    n_seq = n_sparse = n_tie = n_skipped = 0
    for case in range(40):
        rng = np.random.default_rng(47000 + 100 * block + case)
        bf16 = bool(case % 2)
        V = int(rng.choice([1, 2, 3, 7, 8, 17, 64, 300, 1000, 4096, 5001, 20000]))
        B, k = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        z_t, z_d, z_c, _ = _adversarial_rows(rng, B, k, V, bf16)
        zs = dict(t=z_t, d=z_d, c=z_c)
        par = {}
        for name in ("t", "d", "c"):
            T = float(np.float32(rng.choice([1e-3, 0.05, 0.7, 1.0, 1.3, 10.0, 1e3])))
            K = int(rng.choice([0, 1, 2, 5, 20, 50, V]))
            Pp = float(rng.choice([1.0, 0.999, 0.9, 0.5, 0.01]))
            par[name] = (T, K, Pp)
        in_range = True
        for name in ("t", "d", "c"):
            z = zs[name]
            no_mask = np.isfinite(z) & (np.abs(z) < 1e20)
            if no_mask.any() and (np.abs(z[no_mask]) / par[name][0] * 1.4427 > 2 ** 29).any():
                in_range = False
        if not in_range:
            n_skipped += 1
            continue
        s, p, t = _warped_case(rng, zs, torch.bfloat16 if bf16 else torch.float32, par, with_kl=False)
        n_seq, n_sparse, n_tie = n_seq + s, n_sparse + p, n_tie + t
    print(f"\n  adversarial warped block {block}: {n_seq} sequence checks, {n_sparse} compacted pairs, "
          f"near-tie {n_tie}, out of range {n_skipped}", flush=True)
    assert n_seq >= 40 and n_sparse >= 40


def test_flat_companion_row_with_a_wide_support():
    """A case the sweeps above once found: companion logits near 1e4 at temperature 1000 with
    top-p 0.9 (115 384 of 128 256 tokens kept, each with a mass of 8.7e-6).  Bin masses summed
    in fp32 put the cutoff a dozen entries off, which moved S by 1e-4."""
    rng = np.random.default_rng(90086)
    V = int(rng.choice([70000, 152064, 128256, 32000]))
    B, k = int(rng.integers(1, 4)), int(rng.integers(1, 5))
    assert (V, B, k) == (128256, 3, 2)
    z_t, z_d, z_c, _ = _adversarial_rows(rng, B, k, V, False)
    par = {"t": (float(np.float32(1.3)), 2, 0.5), "d": (float(np.float32(1.3)), 20, 0.999), "c": (1000.0, 0, 0.9)}
    n_seq, n_sparse, _ = _warped_case(rng, dict(t=z_t, d=z_d, c=z_c), torch.float32, par, with_kl=False)
    assert n_seq > 0
