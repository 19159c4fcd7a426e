// sv_row_stats: draft/companion indicators of Speculative Verification
// (Sec. 4.2 of the SV paper and the appendix definitions of S and A).
//
// One workgroup per (sequence, position).  Sweep 1 streams the draft row and
// the companion row together with 128-bit loads and keeps one online
// (max, sum-exp) accumulator per row and lane.  S = sum_v min(P_d, P_c) needs
// both normalisers before the element-wise comparison, so a second sweep over
// the pair is unavoidable; it accumulates
//     min(P_d, P_c) = 2^min(a_d, a_c),  a = z * L32 - kappa   (one exp per entry)
// and, on request, KL(P_d || P_c) = ln2 * sum_v P_d (a_d - a_c) and the draft
// entropy H(P_d) = -ln2 * sum_v P_d log2 P_d; the draft's probability of its own
// token, P_d(x), is a free by-product of the epilogue.  (Draft entropy and
// draft-token probability are the signals of the prior acceptance predictors
// discussed in Sec. 2 of the paper.)
// A = min(1, P_c(x) / P_d(x)) is a scalar epilogue in fp64.
//
// Two kernels:
//  * row_stats_stash_kernel (rows on 16-byte boundaries): 512 lanes, two
//    workgroups per CU, so that one's arithmetic overlaps the other's loads.
//    Sweep 1 parks what it reads on chip - the first 10 vector pairs of every
//    lane stay in registers, the next 2432 pairs go to LDS (76 KB) - and only
//    the rest of the pair (about three fifths at V = 152064, bf16) is read
//    again, most recent bytes first so that they are still in L2.
//  * row_stats_kernel: plain two-sweep version for rows of any alignment.
// Algorithmic HBM traffic: 2 * V * elem_size bytes per workgroup.
#include "sv_device.hpp"
#include "sv_host.hpp"

// Phase marks: empty in the library; a profiling build may define
// SV_PHASE_MARK(n) to record a clock at the boundaries of the kernel's phases.
#ifndef SV_PHASE_MARK
#define SV_PHASE_MARK(n)
#endif

namespace sv {

constexpr int kStatsThreads = 1024;

struct StatsArgs {
  const void* z_d;
  const void* z_c;
  const int32_t* x;
  int B, k, V;
  float* lse_d;
  float* lse_c;
  float* S;
  float* A;
  float* kl;          // nullable
  float* entropy_d;   // nullable
  float* pd_x;        // nullable
  uint32_t* flags;    // nullable
  // warped entry point only
  Scale sc_d, sc_c;       // exponent scales (temperatures) of the two tensors
  const float* cut_d;     // nullable: support cutoff of every draft row
  const float* cut_c;     // nullable: support cutoff of every companion row
  // left in the workspace for sv_verify_sample_chained: the draft rows' normalisers
  // and the draft logits of the drafted tokens, under a header that names this call
  ChainHeader* chain;
  double* chain_s;
  float* chain_m;
  float* chain_zx;
  int dtype;
};

// Online sweep of two rows at once (more independent loads in flight).
// WARP: each row has its own exponent scale and support cutoff.
template <int DT, bool WARP>
__device__ __forceinline__ void sweep_online_pair(const void* ra, const void* rb, int V,
                                                  Online& acc_a, Online& acc_b,
                                                  const float La, const float Lb, const float cut_a,
                                                  const float cut_b) {
  constexpr int EPV = Elem<DT>::per_vec;
  const int tid = threadIdx.x, nt = blockDim.x;
  auto add_vec = [&](const u32x4& q, Online& acc, const float L, const float cut) {
    float f[EPV];
    unpack<DT>(q, f);
    if (WARP) {
#pragma unroll
      for (int j = 0; j < EPV; ++j) f[j] = cut_below(f[j], cut);
    }
    acc.add(f, L);
  };
  auto add_one = [&](int v) {
    const float za = load_elem<DT>(ra, v), zb = load_elem<DT>(rb, v);
    acc_a.add1(WARP ? cut_below(za, cut_a) : za, La);
    acc_b.add1(WARP ? cut_below(zb, cut_b) : zb, Lb);
  };
  if (aligned16(ra) && aligned16(rb)) {
    const u32x4* pa = reinterpret_cast<const u32x4*>(ra);
    const u32x4* pb = reinterpret_cast<const u32x4*>(rb);
    const int nvec = V / EPV;
    int i = tid;
    for (; i + nt < nvec; i += 2 * nt) {
      const u32x4 a0 = pa[i], b0 = pb[i], a1 = pa[i + nt], b1 = pb[i + nt];
      add_vec(a0, acc_a, La, cut_a);
      add_vec(b0, acc_b, Lb, cut_b);
      add_vec(a1, acc_a, La, cut_a);
      add_vec(b1, acc_b, Lb, cut_b);
    }
    for (; i < nvec; i += nt) {
      const u32x4 a0 = pa[i], b0 = pb[i];
      add_vec(a0, acc_a, La, cut_a);
      add_vec(b0, acc_b, Lb, cut_b);
    }
    for (int v = nvec * EPV + tid; v < V; v += nt) add_one(v);
  } else {
    for (int v = tid; v < V; v += nt) add_one(v);
  }
}

// Sweep-2 arithmetic for one vocabulary entry (see row_stats_kernel for the
// head/tail split of the normalisers).
template <bool WITH_KL>
struct MinAcc {
  float kd, kc, delta;
  float Ld = kL32, Lc = kL32;          // exponent scales of the two rows
  float acc_s = 0.f, acc_kl = 0.f;
  float acc_pa = 0.f, acc_p = 0.f;     // sum P_d * log2-arg and sum P_d (draft entropy)
  __device__ __forceinline__ void add(float zd, float zc) {
    const float ad = __builtin_fmaf(zd, Ld, -kd);
    const float ac = __builtin_fmaf(zc, Lc, -kc) + delta;
    if (WITH_KL) {
      const float pd = exp2_fast(ad);
      acc_s += fminf(pd, exp2_fast(ac));
      const float t = pd * (ad - ac);          // 0 * inf when P_d underflows: dropped below
      acc_kl += (pd > 0.f) ? t : 0.f;
      const float u = pd * ad;
      acc_pa += (pd > 0.f) ? u : 0.f;
      acc_p += pd;
    } else {
      acc_s += exp2_fast(fminf(ad, ac));
    }
  }
  template <int DT, bool WARP = false>
  __device__ __forceinline__ void add_vec(const u32x4& qd, const u32x4& qc, const float cut_d = -INFINITY,
                                          const float cut_c = -INFINITY) {
    float fd[Elem<DT>::per_vec], fc[Elem<DT>::per_vec];
    unpack<DT>(qd, fd);
    unpack<DT>(qc, fc);
    if (WARP) {
#pragma unroll
      for (int j = 0; j < Elem<DT>::per_vec; ++j) { fd[j] = cut_below(fd[j], cut_d); fc[j] = cut_below(fc[j], cut_c); }
    }
#pragma unroll
    for (int j = 0; j < Elem<DT>::per_vec; ++j) {
      add(fd[j], fc[j]);
      // both sums advance together: otherwise all S terms are formed first and
      // the exponents wait in scratch for the KL terms
      if (WITH_KL && (j & 1)) asm volatile("" : "+v"(acc_s), "+v"(acc_kl), "+v"(acc_pa), "+v"(acc_p));
    }
  }
};

// Scalar epilogue shared by both kernels: A, flags and the stores.
template <int DT, bool WITH_KL, bool WARP = false>
__device__ __forceinline__ void stats_epilogue(const StatsArgs& a, int pair, const void* rd, const void* rc,
                                               double lse_d, double lse_c, double S, double KL, double H_d,
                                               const float cut_d = -INFINITY, const float cut_c = -INFINITY) {
  const bool bad = isnan(lse_d) || isnan(lse_c);
  uint32_t fl = bad ? SV_FLAG_BAD_ROW : 0u;
  double A = __builtin_nan(""), pdx = __builtin_nan("");
  const int tok = a.x[pair];
  const bool tok_ok = tok >= 0 && tok < a.V;
  float zxd = __builtin_nanf("");
  if (tok_ok) {
    zxd = load_elem<DT>(rd, tok);
    if (WARP) zxd = cut_below(zxd, cut_d);
  }
  a.chain_zx[pair] = zxd;                  // whatever the companion row is like
  if (pair == 0) {
    ChainHeader h;
    h.z_d = reinterpret_cast<uint64_t>(a.z_d); h.x = reinterpret_cast<uint64_t>(a.x);
    h.cut_d = WARP ? reinterpret_cast<uint64_t>(a.cut_d) : 0;
    h.B = a.B; h.k = a.k; h.V = a.V; h.dtype = a.dtype;
    h.scale_bits = __float_as_uint(WARP ? a.sc_d.L : kL32);
    h.magic = kChainMagic;
    *a.chain = h;
  }
  if (!bad) {
    if (!tok_ok) {
      fl |= SV_FLAG_BAD_TOKEN;
    } else {
      float zxc = load_elem<DT>(rc, tok);
      double inv_td = 1.0, inv_tc = 1.0;
      if (WARP) {
        zxc = cut_below(zxc, cut_c);
        inv_td = a.sc_d.inv_t; inv_tc = a.sc_c.inv_t;
      }
      const double ld = (double)zxd * inv_td - lse_d;
      const double lc = (double)zxc * inv_tc - lse_c;
      A = (ld == -INFINITY) ? 1.0 : fmin(1.0, exp(lc - ld));
      pdx = exp(ld);
    }
  }
  a.lse_d[pair] = (float)lse_d;
  a.lse_c[pair] = (float)lse_c;
  a.S[pair] = (float)S;
  a.A[pair] = (float)A;
  if (WITH_KL && a.kl) a.kl[pair] = (float)KL;
  if (WITH_KL && a.entropy_d) a.entropy_d[pair] = (float)H_d;
  if (a.pd_x) a.pd_x[pair] = (float)pdx;
  if (a.flags) a.flags[pair] = fl;
}

constexpr int kStashThreads = 512;
constexpr int kLdsVecs = 2432;       // vector pairs parked in LDS (2 * 2432 * 16 B = 76 KB)
constexpr int kLdsIters = (kLdsVecs + kStashThreads - 1) / kStashThreads;
constexpr size_t kStashLdsBytes = 2 * (size_t)kLdsVecs * 16;

// Per-pair constants of sweep 2, formed once (fp64 log2 is ~100 instructions)
// by lanes 0 and 1 of wavefront 0 after the merge and shared through LDS.
struct PairConsts {
  double lse[2];      // natural-log normalisers (NaN: bad row)
  double kappa[2];    // L32-consistent log2 normalisers
};

// Folds the per-wavefront partials left by the first half of block_merge and
// publishes the constants.  Must be called by all threads; ends with a barrier.
__device__ __forceinline__ void publish_pair_consts(const Online (&on)[2], MergeScratch<2>& mg, PairConsts& pc,
                                                    const StatsArgs& a, const int pair,
                                                    const Scale sc_d = unit_scale(), const Scale sc_c = unit_scale()) {
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
#pragma unroll
  for (int r = 0; r < 2; ++r) {
    const float mw = wave_max_f32(on[r].m);
    const float L = r == 0 ? sc_d.L : sc_c.L;
    const double sw = wave_sum_f64((double)on[r].s * (double)exp2_fast(on[r].c - ref_of(mw, L)));
    if ((threadIdx.x & 63) == 0) { mg.m[r][wave] = mw; mg.s[r][wave] = sw; }
  }
  __syncthreads();
  if (threadIdx.x < 2) {
    const int r = threadIdx.x;
    const Scale sc = r == 0 ? sc_d : sc_c;
    const MS ms = fold_parts(mg.m[r], mg.s[r], nw, sc.L);
    pc.lse[r] = lse_from_ms(ms, sc);
    pc.kappa[r] = kappa_l32(ms, sc.L);
    if (r == 0) { a.chain_m[pair] = ms.m; a.chain_s[pair] = ms.s; }
  }
  __syncthreads();
}

// 16 bytes per lane from global memory straight into LDS: lane l of the
// wavefront writes lds_wave_base + 16 * l (global_load_lds_dwordx4).
__device__ __forceinline__ void load_to_lds(const u32x4* src, u32x4* lds_wave_base) {
  __builtin_amdgcn_global_load_lds(
      reinterpret_cast<const __attribute__((address_space(1))) void*>(reinterpret_cast<uintptr_t>(src)),
      reinterpret_cast<__attribute__((address_space(3))) void*>(reinterpret_cast<uintptr_t>(lds_wave_base)),
      16, 0, 0);
}

// vector pairs per lane parked in registers: what fits beside the sweep-2
// arithmetic within the 128 VGPRs that two 512-lane workgroups per CU leave each lane
template <bool WITH_KL>
constexpr int reg_iters() { return WITH_KL ? 8 : 10; }

template <int DT, bool WITH_KL, bool WARP>
__global__ __launch_bounds__(kStashThreads, 4) void row_stats_stash_kernel(StatsArgs a) {
  constexpr int kRegIters = reg_iters<WITH_KL>();
  extern __shared__ u32x4 park[];                      // [kLdsVecs] draft, then [kLdsVecs] companion
  __shared__ BlockScratch sm;
  __shared__ MergeScratch<2> mg;
  __shared__ PairConsts consts;
  constexpr int EPV = Elem<DT>::per_vec;
  constexpr uint32_t kNegInfWord = (DT == DT_BF16) ? 0xFF80FF80u : 0xFF800000u;
  const int tid = threadIdx.x;
  constexpr int nt = kStashThreads;
  const int pair = blockIdx.x;
  const size_t row_bytes = (size_t)a.V * Elem<DT>::bytes;
  const u32x4* pd = reinterpret_cast<const u32x4*>(static_cast<const char*>(a.z_d) + pair * row_bytes);
  const u32x4* pc = reinterpret_cast<const u32x4*>(static_cast<const char*>(a.z_c) + pair * row_bytes);
  const int nvec = a.V / EPV;                           // rows are whole vectors here
  const int lds_begin = kRegIters * nt;
  const int lds_end = min(nvec, lds_begin + kLdsVecs);
  const u32x4 neg = {kNegInfWord, kNegInfWord, kNegInfWord, kNegInfWord};
  Scale sc_d = unit_scale(), sc_c = unit_scale();
  float cut_d = -INFINITY, cut_c = -INFINITY;
  if (WARP) {
    sc_d = a.sc_d; sc_c = a.sc_c;
    if (a.cut_d) cut_d = a.cut_d[pair];
    if (a.cut_c) cut_c = a.cut_c[pair];
  }
  const float Ld = sc_d.L, Lc = sc_c.L;
  // sweep-1 step for one vector of one row
  auto add1 = [&](Online& o, const u32x4& q, const float L, const float cut) {
    float f[EPV];
    unpack<DT>(q, f);
    if (WARP) {
#pragma unroll
      for (int j = 0; j < EPV; ++j) f[j] = cut_below(f[j], cut);
    }
    o.add(f, L);
  };

  // ---- sweep 1 ------------------------------------------------------------
  SV_PHASE_MARK(0)
  Online on[2];
  Online& od = on[0];
  Online& oc = on[1];
  od.init();
  oc.init();
  u32x4 sd[kRegIters], sc[kRegIters];
#pragma unroll
  for (int j = 0; j < kRegIters; ++j) {                 // all loads in flight before any use
    const int i = tid + j * nt;
    sd[j] = neg;
    sc[j] = neg;
    if (i < nvec) { sd[j] = __builtin_nontemporal_load(pd + i); sc[j] = __builtin_nontemporal_load(pc + i); }
  }
  // the LDS share goes straight from memory into LDS (no registers in between)
  // and lands while the register share is being accumulated
  {
    const int wave_base = tid & ~(kWave - 1);
#pragma unroll
    for (int j = 0; j < kLdsIters; ++j) {
      const int slot = j * nt + wave_base;              // LDS slot of lane 0; the hardware adds lane * 16 B
      const int i = lds_begin + j * nt + tid;
      if (i < lds_end) {
        load_to_lds(pd + i, park + slot);
        load_to_lds(pc + i, park + kLdsVecs + slot);
      }
    }
  }
  SV_PHASE_MARK(1)
#pragma unroll
  for (int j = 0; j < kRegIters; ++j) {                 // -inf padding adds nothing
    add1(od, sd[j], Ld, cut_d);
    __builtin_amdgcn_sched_barrier(0);
    add1(oc, sc[j], Lc, cut_c);
    __builtin_amdgcn_sched_barrier(0);                  // one pair at a time: the parked vectors own the registers
  }
  SV_PHASE_MARK(2)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // LDS share has landed (own lanes only: no barrier)
  for (int i = lds_begin + tid; i < lds_end; i += nt) {
    add1(od, park[i - lds_begin], Ld, cut_d);
    add1(oc, park[kLdsVecs + i - lds_begin], Lc, cut_c);
  }
  SV_PHASE_MARK(3)
  {
    int i = lds_end + tid;
    for (; i + nt < nvec; i += 2 * nt) {
      const u32x4 d0 = pd[i], c0 = pc[i], d1 = pd[i + nt], c1 = pc[i + nt];
      add1(od, d0, Ld, cut_d);
      __builtin_amdgcn_sched_barrier(0);
      add1(oc, c0, Lc, cut_c);
      __builtin_amdgcn_sched_barrier(0);
      add1(od, d1, Ld, cut_d);
      __builtin_amdgcn_sched_barrier(0);
      add1(oc, c1, Lc, cut_c);
      __builtin_amdgcn_sched_barrier(0);
    }
    for (; i < nvec; i += nt) {
      const u32x4 d0 = pd[i], c0 = pc[i];
      add1(od, d0, Ld, cut_d);
      add1(oc, c0, Lc, cut_c);
    }
  }
  SV_PHASE_MARK(4)
  publish_pair_consts(on, mg, consts, a, pair, sc_d, sc_c);
  const double lse_d = consts.lse[0], lse_c = consts.lse[1];
  const bool bad = isnan(lse_d) || isnan(lse_c);

  SV_PHASE_MARK(5)
  // ---- sweep 2: rest of the pair from L2/HBM (newest first), then LDS, then registers
  double S = __builtin_nan(""), KL = __builtin_nan(""), H_d = __builtin_nan("");
  if (!bad) {
    const double kappa_d = consts.kappa[0], kappa_c = consts.kappa[1];
    MinAcc<WITH_KL> acc;
    acc.kd = (float)kappa_d;
    acc.kc = (float)kappa_c;
    const double tail_d = kappa_d - (double)acc.kd, tail_c = kappa_c - (double)acc.kc;
    acc.delta = (float)(tail_d - tail_c);
    acc.Ld = Ld; acc.Lc = Lc;
    {
      // walk the re-read region backwards: its end was read last in sweep 1
      const int n_rest = nvec - lds_end;
      int r = tid;
      for (; r + nt < n_rest; r += 2 * nt) {
        const int i0 = nvec - 1 - r, i1 = nvec - 1 - (r + nt);
        const u32x4 d0 = __builtin_nontemporal_load(pd + i0), c0 = __builtin_nontemporal_load(pc + i0),
                    d1 = __builtin_nontemporal_load(pd + i1), c1 = __builtin_nontemporal_load(pc + i1);
        acc.template add_vec<DT, WARP>(d0, c0, cut_d, cut_c);
        __builtin_amdgcn_sched_barrier(0);
        acc.template add_vec<DT, WARP>(d1, c1, cut_d, cut_c);
        __builtin_amdgcn_sched_barrier(0);
      }
      for (; r < n_rest; r += nt) {
        const int i0 = nvec - 1 - r;
        acc.template add_vec<DT, WARP>(pd[i0], pc[i0], cut_d, cut_c);
      }
    }
    SV_PHASE_MARK(6)
    for (int i = lds_begin + tid; i < lds_end; i += nt)
      acc.template add_vec<DT, WARP>(park[i - lds_begin], park[kLdsVecs + i - lds_begin], cut_d, cut_c);
    SV_PHASE_MARK(7)
#pragma unroll
    for (int j = 0; j < kRegIters; ++j) {               // -inf padding: 2^-inf = 0
      // keep the vectors packed between the sweeps: without this the unpacked
      // floats of sweep 1 are kept alive for reuse and spill
      asm volatile("" : "+v"(sd[j].x), "+v"(sd[j].y), "+v"(sd[j].z), "+v"(sd[j].w));
      asm volatile("" : "+v"(sc[j].x), "+v"(sc[j].y), "+v"(sc[j].z), "+v"(sc[j].w));
      acc.template add_vec<DT, WARP>(sd[j], sc[j], cut_d, cut_c);
      __builtin_amdgcn_sched_barrier(0);
    }
    SV_PHASE_MARK(8)
    S = block_sum_f64((double)acc.acc_s, sm);
    if (WITH_KL) {
      KL = block_sum_f64((double)acc.acc_kl, sm);
      const double pa = block_sum_f64((double)acc.acc_pa, sm), p1 = block_sum_f64((double)acc.acc_p, sm);
      H_d = pa - tail_d * p1;                  // sum 2^(a_d) * log2 P_d, still without f_d
    }
    if (tid == 0) {
      const double f_d = exp2(-tail_d);
      S *= f_d;
      KL *= f_d * kLn2;
      H_d *= -f_d * kLn2;
    }
  }
  SV_PHASE_MARK(9)
  if (tid == 0) stats_epilogue<DT, WITH_KL, WARP>(a, pair, pd, pc, lse_d, lse_c, S, KL, H_d, cut_d, cut_c);
}

template <int DT, bool WITH_KL, bool WARP>
__global__ __launch_bounds__(kStatsThreads) void row_stats_kernel(StatsArgs a) {
  __shared__ BlockScratch sm;
  __shared__ MergeScratch<2> mg;
  __shared__ PairConsts consts;
  const int pair = blockIdx.x;                       // b * k + i
  const size_t row_bytes = (size_t)a.V * Elem<DT>::bytes;
  const void* rd = static_cast<const char*>(a.z_d) + pair * row_bytes;
  const void* rc = static_cast<const char*>(a.z_c) + pair * row_bytes;

  Scale sc_d = unit_scale(), sc_c = unit_scale();
  float cut_d = -INFINITY, cut_c = -INFINITY;
  if (WARP) {
    sc_d = a.sc_d; sc_c = a.sc_c;
    if (a.cut_d) cut_d = a.cut_d[pair];
    if (a.cut_c) cut_c = a.cut_c[pair];
  }
  Online on[2];
  on[0].init();
  on[1].init();
  sweep_online_pair<DT, WARP>(rd, rc, a.V, on[0], on[1], sc_d.L, sc_c.L, cut_d, cut_c);
  publish_pair_consts(on, mg, consts, a, pair, sc_d, sc_c);
  const double lse_d = consts.lse[0], lse_c = consts.lse[1];
  const bool bad = isnan(lse_d) || isnan(lse_c);

  double S = __builtin_nan(""), KL = __builtin_nan(""), H_d = __builtin_nan("");
  if (!bad) {
    // kappa = log2-domain normaliser consistent with the L32 exponent scale,
    // split into an fp32 head and a tail.  With a = z*L32 - head:
    // P_d = f_d 2^(a_d),  P_c = f_d 2^(a_c + delta),
    // f_d = 2^(-tail_d), delta = tail_d - tail_c, so one scalar factor at the
    // end removes the rounding of both heads.
    const double kappa_d = consts.kappa[0], kappa_c = consts.kappa[1];
    MinAcc<WITH_KL> acc;
    acc.kd = (float)kappa_d;
    acc.kc = (float)kappa_c;
    const double tail_d = kappa_d - (double)acc.kd, tail_c = kappa_c - (double)acc.kc;
    acc.delta = (float)(tail_d - tail_c);
    acc.Ld = sc_d.L; acc.Lc = sc_c.L;
    visit_range<DT, true>(rd, rc, 0, a.V, [&](int, float zd, float zc) {
      if (WARP) { zd = cut_below(zd, cut_d); zc = cut_below(zc, cut_c); }
      acc.add(zd, zc);
    });
    S = block_sum_f64((double)acc.acc_s, sm);
    if (WITH_KL) {
      KL = block_sum_f64((double)acc.acc_kl, sm);
      const double pa = block_sum_f64((double)acc.acc_pa, sm), p1 = block_sum_f64((double)acc.acc_p, sm);
      H_d = pa - tail_d * p1;
    }
    if (threadIdx.x == 0) {
      const double f_d = exp2(-tail_d);
      S *= f_d;
      KL *= f_d * kLn2;
      H_d *= -f_d * kLn2;
    }
  }
  if (threadIdx.x == 0)
    stats_epilogue<DT, WITH_KL, WARP>(a, pair, rd, rc, lse_d, lse_c, S, KL, H_d, cut_d, cut_c);
}

template <int DT, bool WITH_KL, bool WARP>
static int launch_stats(const StatsArgs& a, bool rows_aligned, hipStream_t st) {
  const dim3 grid(a.B * a.k);
  if (rows_aligned) {
    // more than 64 KB of dynamic LDS has to be allowed once per kernel and device
    constexpr int kMaxDevices = 64;
    static bool allowed[kMaxDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SV_ERR_LAUNCH;
    if (dev < 0 || dev >= kMaxDevices || !allowed[dev]) {
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(&row_stats_stash_kernel<DT, WITH_KL, WARP>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStashLdsBytes) != hipSuccess)
        return SV_ERR_LAUNCH;
      if (dev >= 0 && dev < kMaxDevices) allowed[dev] = true;
    }
    TapScope tap(SV_KERNEL_ROW_STATS, st);
    hipLaunchKernelGGL((row_stats_stash_kernel<DT, WITH_KL, WARP>), grid, dim3(kStashThreads), kStashLdsBytes, st, a);
  } else {
    TapScope tap(SV_KERNEL_ROW_STATS, st);
    hipLaunchKernelGGL((row_stats_kernel<DT, WITH_KL, WARP>), grid, dim3(kStatsThreads), 0, st, a);
  }
  return launch_status();
}

// Argument checks and launch shared by sv_row_stats and sv_row_stats_warped.
static int row_stats_checked(const void* z_d, const void* z_c, const int32_t* x, int B, int k, int V, int dtype,
                             bool warped, const Scale& sc_d, const float* cut_d, const Scale& sc_c,
                             const float* cut_c, float* lse_d, float* lse_c, float* S, float* A, float* kl,
                             float* entropy_d, float* pd_x, uint32_t* flags, void* ws, size_t ws_bytes,
                             sv_stream_t stream) {
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE((long long)B * k <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(z_d && z_c && x && lse_d && lse_c && S && A, SV_ERR_NULL);
  const int eb = elem_bytes(dtype);
  SV_REQUIRE(is_aligned(z_d, eb) && is_aligned(z_c, eb), SV_ERR_ALIGN);
  SV_REQUIRE(is_aligned(x, 4) && is_aligned(lse_d, 4) && is_aligned(lse_c, 4) && is_aligned(S, 4) &&
                 is_aligned(A, 4) && is_aligned(kl, 4) && is_aligned(entropy_d, 4) && is_aligned(pd_x, 4) &&
                 is_aligned(flags, 4) && is_aligned(cut_d, 4) && is_aligned(cut_c, 4),
             SV_ERR_ALIGN);
  SV_REQUIRE(ws && is_aligned(ws, kWsAlign) && ws_bytes >= sv_workspace_bytes(B, k, V, dtype),
             SV_ERR_WORKSPACE);
  const VerifyWs w = carve_verify_ws(ws, B, k, V);
  StatsArgs a{z_d, z_c, x, B, k, V, lse_d, lse_c, S, A, kl, entropy_d, pd_x, flags, sc_d, sc_c, cut_d, cut_c,
              w.chain, w.chain_s, w.chain_m, w.chain_zx, dtype};
  const bool extended = kl || entropy_d;   // sums that need P_d of every entry
  const bool rows_aligned = is_aligned(z_d, 16) && is_aligned(z_c, 16) && ((size_t)V * eb) % 16 == 0;
  hipStream_t st = as_stream(stream);
  if (warped) {
    if (dtype == SV_F32)
      return extended ? launch_stats<DT_F32, true, true>(a, rows_aligned, st)
                      : launch_stats<DT_F32, false, true>(a, rows_aligned, st);
    return extended ? launch_stats<DT_BF16, true, true>(a, rows_aligned, st)
                    : launch_stats<DT_BF16, false, true>(a, rows_aligned, st);
  }
  if (dtype == SV_F32)
    return extended ? launch_stats<DT_F32, true, false>(a, rows_aligned, st)
                    : launch_stats<DT_F32, false, false>(a, rows_aligned, st);
  return extended ? launch_stats<DT_BF16, true, false>(a, rows_aligned, st)
                  : launch_stats<DT_BF16, false, false>(a, rows_aligned, st);
}

}  // namespace sv

extern "C" int sv_row_stats(const void* z_d, const void* z_c, const int32_t* x,
                            int B, int k, int V, int dtype,
                            float* lse_d, float* lse_c, float* S, float* A,
                            float* kl_or_null, float* entropy_d_or_null, float* pd_x_or_null,
                            uint32_t* flags_or_null,
                            void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  return row_stats_checked(z_d, z_c, x, B, k, V, dtype, false, unit_scale(), nullptr, unit_scale(), nullptr,
                           lse_d, lse_c, S, A, kl_or_null, entropy_d_or_null, pd_x_or_null, flags_or_null, ws,
                           ws_bytes, stream);
}

extern "C" int sv_row_stats_warped(const void* z_d, const void* z_c, const int32_t* x,
                                   int B, int k, int V, int dtype,
                                   float temperature_d, const float* cutoff_d_or_null,
                                   float temperature_c, const float* cutoff_c_or_null,
                                   float* lse_d, float* lse_c, float* S, float* A,
                                   float* kl_or_null, float* entropy_d_or_null, float* pd_x_or_null,
                                   uint32_t* flags_or_null,
                                   void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  Scale sc_d, sc_c;
  SV_REQUIRE(scale_of(temperature_d, &sc_d) && scale_of(temperature_c, &sc_c), SV_ERR_INVALID_ARG);
  return row_stats_checked(z_d, z_c, x, B, k, V, dtype, true, sc_d, cutoff_d_or_null, sc_c, cutoff_c_or_null,
                           lse_d, lse_c, S, A, kl_or_null, entropy_d_or_null, pd_x_or_null, flags_or_null, ws,
                           ws_bytes, stream);
}
