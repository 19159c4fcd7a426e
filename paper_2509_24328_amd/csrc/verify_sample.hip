// sv_verify_sample: speculative-sampling verification of the selected draft
// prefix of every sequence (Sec. 4.2 last paragraph of the SV paper; the
// accept / residual / bonus rule is the standard speculative-sampling one).
//
// Three kernels on the caller's stream:
//
//  1. verify_rows_kernel   1..8 workgroups per logit row that the step needs
//     (target rows 0..gamma_b, draft rows 0..gamma_b-1 of every sequence).
//     Each streams its part of the row once with 128-bit loads and keeps a
//     per-lane online (max, sum-exp); writes the part's (m, s) and the logit
//     of the drafted token.  Rows outside the verification length exit without
//     reading.  HBM-bound: V * elem_size bytes per row.
//
//  2. verify_mass_kernel   grid (chunks, B).  First the accept decision of the
//     sequence, by one wavefront with one lane per drafted position (k <= 64):
//     folds the row partials, forms the acceptance ratios in fp64, draws the
//     Philox uniforms and counts the leading accepts.  Every workgroup of a
//     sequence does this for itself (a few hundred bytes and two fp64
//     logarithms: less than a kernel boundary costs); the one of chunk 0 writes
//     the accepted tokens and the plan of the sampling stage.  Then the
//     workgroup sums its 8192-entry chunk of the sampling row: residual
//     max(0, P_t - P_d) and P_t.  Touches B rows (pairs).
//
//  3. verify_pick_kernel   one workgroup per sequence: scans the chunk masses in
//     order (fp64), locates the chunk holding u' * W, stages that chunk's
//     weights in LDS and finds the token with a block prefix scan.
//
// Kernel boundaries carry the cross-workgroup hand-offs (row scalars, plan,
// chunk masses): device-scope fences inside a kernel were measured to cost far
// more than a launch on this part.
#include <algorithm>
#include <mutex>

#include "sv_device.hpp"
#include "sv_host.hpp"

// Phase marks: empty in the library; a profiling build may define
// SV_PHASE_MARK(n) to record a clock at the boundaries of a kernel's phases.
#ifndef SV_PHASE_MARK
#define SV_PHASE_MARK(n)
#endif

namespace sv {

constexpr int kRowsThreads = 256;
constexpr int kSampleThreads = 256;             // mass kernel: one workgroup per chunk
constexpr int kPickThreads = 1024;              // pick kernel: one workgroup per sequence
constexpr int kMaxChunks = 2048;                // V <= kMaxChunks * kChunk
static_assert(kMaxSplit == kMaxParts, "fold_row_parts reads up to kMaxParts partials of a row");

struct VerifyArgs {
  const void* z_t;
  const int32_t* t_offsets;   // nullable
  int n_t_rows;
  const void* z_d;
  const int32_t* x;
  const int32_t* gamma;       // nullable
  int B, k, V;
  int split;                  // workgroups per row in verify_rows_kernel
  int t_seq_rows;             // rows per sequence of a dense z_t (k + 1, or k without bonus rows)
  int with_bonus;             // 0: target row gamma_b (bonus position) is not needed
  uint32_t seed_lo, seed_hi, step;
  int32_t* out_tokens;
  int32_t* n_accept;
  uint32_t* flags;
  float* ratio;               // nullable
  Scale sc_t, sc_d;           // exponent scales (temperatures) of the two tensors
  const float* cut_t;         // nullable: support cutoff of every row of z_t
  const float* cut_d;         // nullable: support cutoff of every row of z_d
  int chained;                // 1: draft normalisers come from the statistics pass (workspace), z_d's rows
                              // are not swept
  int dtype;
  VerifyWs ws;
};

__device__ __forceinline__ int gamma_of(const VerifyArgs& a, int b) {
  int g = a.gamma ? a.gamma[b] : a.k;
  return min(max(g, 0), a.k);
}

// Row number in z_t of target position (b, i), or -1 when a packed offset
// points outside z_t.
__device__ __forceinline__ long target_index(const VerifyArgs& a, int b, int i) {
  if (a.t_offsets) {
    const long row = (long)a.t_offsets[b] + i;
    return (row < 0 || row >= a.n_t_rows) ? -1 : row;
  }
  return (long)b * a.t_seq_rows + i;
}

// Target row of (b, i), or nullptr when a packed offset points outside z_t.
template <int DT>
__device__ __forceinline__ const void* target_row(const VerifyArgs& a, int b, int i) {
  const long row = target_index(a, b, i);
  if (row < 0) return nullptr;
  return static_cast<const char*>(a.z_t) + (size_t)row * a.V * Elem<DT>::bytes;
}

// Support cutoffs of the warped entry point (-inf: the whole vocabulary).
__device__ __forceinline__ float target_cut(const VerifyArgs& a, int b, int i) {
  const long row = target_index(a, b, i);
  return (a.cut_t && row >= 0) ? a.cut_t[row] : -INFINITY;
}
__device__ __forceinline__ float draft_cut(const VerifyArgs& a, int b, int i) {
  return a.cut_d ? a.cut_d[b * a.k + i] : -INFINITY;
}

template <int DT>
__device__ __forceinline__ const void* draft_row(const VerifyArgs& a, int b, int i) {
  return static_cast<const char*>(a.z_d) + ((size_t)b * a.k + i) * a.V * Elem<DT>::bytes;
}

// Normaliser of a whole row from the partials its workgroups left.
__device__ __forceinline__ MS target_ms(const VerifyArgs& a, int b, int i) {
  const int idx = (b * (a.k + 1) + i) * a.split;
  return fold_row_parts(a.ws.m_t + idx, a.ws.s_t + idx, a.split, a.sc_t.L);
}
// Chained calls: does the workspace hold the draft normalisers of this very step?  (The
// header names the tensors, shape and scale the statistics pass was given; what the
// tensors contain is the caller's business.)
__device__ __forceinline__ bool chain_matches(const VerifyArgs& a) {
  // the whole header in three 128-bit loads, compared without short-circuit: field-by-field
  // loads inside a chain of && become as many dependent trips to memory
  static_assert(sizeof(ChainHeader) == 48, "three 16-byte words");
  const u32x4* w = reinterpret_cast<const u32x4*>(a.ws.chain);
  const u32x4 w0 = w[0], w1 = w[1], w2 = w[2];
  const uint64_t zd = reinterpret_cast<uint64_t>(a.z_d), x = reinterpret_cast<uint64_t>(a.x),
                 cd = reinterpret_cast<uint64_t>(a.cut_d);
  uint32_t diff = (w0.x ^ (uint32_t)zd) | (w0.y ^ (uint32_t)(zd >> 32)) | (w0.z ^ (uint32_t)x) |
                  (w0.w ^ (uint32_t)(x >> 32));
  diff |= (w1.x ^ (uint32_t)cd) | (w1.y ^ (uint32_t)(cd >> 32)) | (w1.z ^ (uint32_t)a.B) | (w1.w ^ (uint32_t)a.k);
  diff |= (w2.x ^ (uint32_t)a.V) | (w2.y ^ (uint32_t)a.dtype) | (w2.z ^ __float_as_uint(a.sc_d.L)) |
          (w2.w ^ kChainMagic);
  return diff == 0;
}
__device__ __forceinline__ MS draft_ms(const VerifyArgs& a, int b, int i) {
  const int idx = (b * a.k + i) * a.split;
  return fold_row_parts(a.ws.m_d + idx, a.ws.s_d + idx, a.split, a.sc_d.L);
}

// ---------------------------------------------------------------------------
// kernel 1: row normalisers
// ---------------------------------------------------------------------------
// What one workgroup of the row sweep is about and what it found.
struct RowPart {
  int b, i, part;
  bool is_target, needed;
  MS ms;          // (m, s) of this part of the row
  float zx;       // logit of the drafted token (part 0 of rows i < k), else NaN
};

// The sweep of one part of one needed row by the whole workgroup (results in thread 0).
template <int DT, bool CUT>
__device__ __forceinline__ RowPart sweep_row_part(const VerifyArgs& a, MergeScratch<1>& sm) {
  RowPart r;
  const int per_seq = a.chained ? a.k + 1 : 2 * a.k + 1;       // chained: target rows only
  const int slot = blockIdx.x / a.split;
  r.part = blockIdx.x - slot * a.split;
  r.b = slot / per_seq;
  const int q = slot - r.b * per_seq;
  r.is_target = q <= a.k;
  r.i = r.is_target ? q : q - (a.k + 1);
  const int g = gamma_of(a, r.b);
  r.needed = r.i < (r.is_target ? g + a.with_bonus : g);
  r.zx = __builtin_nanf("");
  if (!r.needed) return r;                               // no bytes read

  const void* row = r.is_target ? target_row<DT>(a, r.b, r.i) : draft_row<DT>(a, r.b, r.i);
  const float L = r.is_target ? a.sc_t.L : a.sc_d.L;
  float cut = -INFINITY;
  if (CUT) cut = r.is_target ? target_cut(a, r.b, r.i) : draft_cut(a, r.b, r.i);
  Online acc[1];
  acc[0].init();
  // six vectors in flight per lane: a part is 8-10 vectors per lane at the benchmark shapes, i.e. two
  // round trips to memory (6 + the rest, whose loads also go out together) instead of three or four
  if (row) sweep_online<DT, CUT, true, 6>(row, a.V, r.part, a.split, acc[0], L, cut);
  MS merged[1];
  block_merge<1>(acc, sm, merged, L);
  r.ms = merged[0];                                      // s = 0 for a missing row => bad row
  if (threadIdx.x == 0 && r.part == 0 && r.i < a.k && row) {
    const int tok = a.x[r.b * a.k + r.i];
    if (tok >= 0 && tok < a.V) r.zx = load_elem<DT>(row, tok);
    if (CUT) r.zx = cut_below(r.zx, cut);
  }
  return r;
}

// Thread 0 leaves the part's results in the workspace.
__device__ __forceinline__ void store_row_part(const VerifyArgs& a, const RowPart& r) {
  if (r.is_target) {
    const int idx = (r.b * (a.k + 1) + r.i) * a.split + r.part;
    a.ws.m_t[idx] = r.ms.m;
    a.ws.s_t[idx] = r.ms.s;
    if (r.part == 0 && r.i < a.k) a.ws.zx_t[r.b * a.k + r.i] = r.zx;
  } else {
    const int idx = (r.b * a.k + r.i) * a.split + r.part;
    a.ws.m_d[idx] = r.ms.m;
    a.ws.s_d[idx] = r.ms.s;
    if (r.part == 0) a.ws.zx_d[r.b * a.k + r.i] = r.zx;
  }
}

template <int DT, bool CUT>
__global__ __launch_bounds__(kRowsThreads) void verify_rows_kernel(VerifyArgs a) {
  __shared__ MergeScratch<1> sm;
  const RowPart r = sweep_row_part<DT, CUT>(a, sm);
  if (r.needed && threadIdx.x == 0) store_row_part(a, r);
}

// ---------------------------------------------------------------------------
// kernel 2: accept count, chunk masses, token
// ---------------------------------------------------------------------------
// Probability of one vocabulary entry: 2^(z l - kappa) with l = log2(e) / T
// carried as L + l_lo and kappa = k_hi + k_lo, so that neither the rounding of
// the scale nor that of the row normaliser biases every entry of a row the
// same way.  The exponent is head + tail, head = z L - k_hi (one fused
// multiply-add: exact up to its own rounding whatever the size of z) and
// tail = z l_lo - k_lo (|tail| grows with |z|: 1e-6 for ordinary logits, 1e-2
// at |z| = 1e6).  2^(head + tail) is formed as 2^a (1 + ln2 r) with
// a = fl(head + tail) and r = what that addition dropped, so the error does
// not grow with the size of the logits.
struct ProbRow {
  float L;         // fl32(log2(e) / T)
  float k_hi;      // fl32(kappa)
  float l_lo;      // log2(e) / T - L
  float k_lo;      // kappa - k_hi
  __device__ __forceinline__ void set(double lse, const Scale& sc) {
    const double kappa = lse * kLog2e;
    L = sc.L;
    k_hi = (float)kappa;
    l_lo = (float)sc.l_lo;
    k_lo = (float)(kappa - (double)k_hi);
  }
  __device__ __forceinline__ float p(float z) const {
    const float head = __builtin_fmaf(z, L, -k_hi);
    const float tail = __builtin_fmaf(z, l_lo, -k_lo);
    const float a = head + tail;
    const float r = (head - a) + tail;
    const float e = exp2_fast(a);
    return e > 0.f ? __builtin_fmaf(e, (float)kLn2 * r, e) : 0.f;   // z = -inf: a is -inf or NaN, mass is 0
  }
};

// grid (B), one wavefront: p_t(x)/p_d(x) of EVERY drafted position (profiling
// pass: no early stop, no sampling), from the row partials of verify_rows_kernel.
__global__ __launch_bounds__(kWave) void accept_ratio_kernel(VerifyArgs a, float* ratio, uint32_t* flags) {
  const int b = blockIdx.x, k = a.k;
  for (int i = threadIdx.x; i < k; i += kWave) {
    uint32_t fl = 0;
    double rho = __builtin_nan("");
    const int tok = a.x[b * k + i];
    if (tok < 0 || tok >= a.V) {
      fl |= SV_FLAG_BAD_TOKEN;
    } else {
      const double lse_t = lse_from_ms(target_ms(a, b, i), a.sc_t), lse_d = lse_from_ms(draft_ms(a, b, i), a.sc_d);
      if (isnan(lse_t) || isnan(lse_d)) {
        fl |= SV_FLAG_BAD_ROW;
      } else {
        const double lt = (double)a.ws.zx_t[b * k + i] * a.sc_t.inv_t - lse_t;
        const double ld = (double)a.ws.zx_d[b * k + i] * a.sc_d.inv_t - lse_d;
        rho = exp(lt - ld);
      }
    }
    ratio[b * k + i] = (float)rho;
    if (flags) flags[b * k + i] = fl;
  }
}

// What the sampling stage needs to know about a sequence, written by the accept kernel.
struct alignas(16) Plan {
  double lse_t, lse_d;
  int n;               // accepted count = position that is sampled
  uint32_t flags;
  int resid;           // 1: residual max(0, P_t - P_d), 0: target distribution
  int target_ok;
};

static_assert(sizeof(Plan) == 32, "workspace carve-up reserves 32 bytes per sequence");

// Accept count of sequence b in fp64, its flags, and the plan for the sampling
// stage.  Run by one whole wavefront (lane i = drafted position i, k <= 64);
// every workgroup of the mass kernel that works on sequence b calls it and gets
// the same plan, the one with `publish` set also writes the accepted tokens,
// the ratios, the accept count and the plan itself for the pick kernel.
template <int DT, bool CHAIN>
__device__ __forceinline__ void accept_plan(const VerifyArgs& a, const int b, const int i, const bool publish,
                                            Plan* plan_out) {
  const int k = a.k, V = a.V;
  const int g = gamma_of(a, b);
  const bool evaluated = i < g;
  bool accept = true;
  uint32_t fl = 0;
  double rho = __builtin_nan("");
  double lse_t = __builtin_nan(""), lse_d = __builtin_nan("");
  bool have_target = false;
  // chained: everything the statistics pass left goes into flight at once, before any branch
  // (three dependent round trips to memory otherwise: header, normaliser, logit)
  bool chain_ok = true;
  MS chain_ms;
  float chain_zx = 0.f;
  if (CHAIN) {
    const int at = b * k + min(i, k - 1);
    chain_ms.m = a.ws.chain_m[at];
    chain_ms.s = a.ws.chain_s[at];
    chain_zx = a.ws.chain_zx[at];
    chain_ok = chain_matches(a);
    if (!chain_ok) { chain_ms.m = -INFINITY; chain_ms.s = 0.0; }   // no sum: an unusable row
  }
  // Everything the decision may need is asked for here, for every lane and before the length is
  // known (rows past the length hold whatever an earlier call left: read, never used), so that
  // the loads travel together instead of in three dependent rounds: length, partials, logits.
  const int it = min(i, k), id = min(i, k - 1);
  const MS ms_t = target_ms(a, b, it);
  const MS ms_d = CHAIN ? chain_ms : draft_ms(a, b, id);
  const float zx_t = a.ws.zx_t[b * k + id];
  const float zx_d = CHAIN ? chain_zx : a.ws.zx_d[b * k + id];
  const int tok = a.x[b * k + id];
  const bool target_there = target_index(a, b, it) >= 0;
  if (i <= g) {                                   // target rows 0..g (row g: bonus position)
    have_target = target_there;
    lse_t = lse_from_ms(ms_t, a.sc_t);
  }
  if (evaluated) {
    lse_d = lse_from_ms(ms_d, a.sc_d);
    if (tok < 0 || tok >= V) {
      fl |= SV_FLAG_BAD_TOKEN;
    } else if (isnan(lse_t) || isnan(lse_d)) {
      fl |= SV_FLAG_BAD_ROW;
    } else {
      const double lt = (double)zx_t * a.sc_t.inv_t - lse_t;
      const double ld = (double)zx_d * a.sc_d.inv_t - lse_d;
      rho = exp(lt - ld);                         // -inf - -inf = NaN: rejected
    }
    const U4 r = philox4x32_10((uint32_t)i, (uint32_t)b, 0u, a.step, a.seed_lo, a.seed_hi);
    const double u = unit_from_word(r.w[0]);
    accept = u < rho;                             // false for NaN
    if (!isnan(rho) && fabs(u - fmin(1.0, rho)) < 1e-6) fl |= SV_FLAG_NEAR_TIE;
  }
  const unsigned long long rej = __ballot(evaluated && !accept);
  const int n = rej ? (int)__builtin_ctzll(rej) : g;          // leading accepts
  // flags of the positions that were actually evaluated: 0..min(n, g-1)
  if (!(evaluated && i <= n)) fl = 0;
  for (int off = 32; off >= 1; off >>= 1) fl |= __shfl_xor(fl, off, kWave);
  if (publish) {
    if (a.ratio && i < k) a.ratio[b * k + i] = (evaluated && i <= n) ? (float)rho : __builtin_nanf("");
    int32_t* out = a.out_tokens + (size_t)b * (k + 1);
    for (int j = i; j <= k; j += kWave) out[j] = (j < n) ? a.x[b * k + j] : -1;
  }
  // the plan of position n, from the values of lane n (position n = 64, the bonus
  // row of a fully accepted k = 64, has no lane: lane 0 forms them itself)
  double lse_t_n, lse_d_n;
  int have_target_n;
  if (n < kWave) {
    lse_t_n = __shfl(lse_t, n, kWave);
    lse_d_n = __shfl(lse_d, n, kWave);
    have_target_n = __shfl((int)have_target, n, kWave);
  } else {
    lse_t_n = lse_from_ms(target_ms(a, b, n), a.sc_t);
    lse_d_n = __builtin_nan("");
    have_target_n = target_row<DT>(a, b, n) != nullptr;
  }
  if (i == 0) {
    uint32_t flags = fl;
    bool resid = n < g;
    const bool target_ok = have_target_n && !isnan(lse_t_n);
    if (resid && isnan(lse_d_n)) {                // unusable draft row: draw from the target instead
      resid = false;
      flags |= SV_FLAG_BAD_ROW | SV_FLAG_RESIDUAL_FALLBACK;
    }
    if (!target_ok) flags |= SV_FLAG_BAD_ROW;
    if (CHAIN && !chain_ok) flags |= SV_FLAG_NO_CHAIN;
    Plan pl;
    pl.lse_t = lse_t_n; pl.lse_d = resid ? lse_d_n : 0.0; pl.n = n; pl.flags = flags;
    pl.resid = resid ? 1 : 0; pl.target_ok = target_ok ? 1 : 0;
    *plan_out = pl;
    if (publish) {
      a.ws.plan[b] = pl;
      a.n_accept[b] = n;
    }
  }
}

// Residual and target mass of chunk c of the sampling row of sequence b, by the whole
// workgroup (results in every thread).  fp64 sums of the fp32 weights: the pick stage forms
// the same weights again and adds them in another order, and the two must agree far inside
// the band of SV_FLAG_NEAR_CDF_EDGE.
template <int DT, bool CUT>
__device__ __forceinline__ void chunk_masses(const VerifyArgs& a, int b, const Plan& pl, int c, BlockScratch& red,
                                             double* mass_r, double* mass_t) {
  const int n = pl.n;
  const bool target_ok = pl.target_ok != 0, resid = pl.resid != 0;
  const void* row_t = target_row<DT>(a, b, n);
  const void* row_d = resid ? draft_row<DT>(a, b, n) : nullptr;
  ProbRow pt, pd;
  pt.set(target_ok ? pl.lse_t : 0.0, a.sc_t);
  pd.set(pl.lse_d, a.sc_d);
  float cut_t = -INFINITY, cut_d = -INFINITY;
  if (CUT) { cut_t = target_cut(a, b, n); if (resid) cut_d = draft_cut(a, b, n); }
  const int v0 = c * kChunk, v1 = min(a.V, v0 + kChunk);
  double acc_r = 0.0, acc_t = 0.0;
  if (target_ok) {
    if (resid) {
      visit_range<DT, true, 4>(row_t, row_d, v0, v1, [&](int, float zt, float zd) {
        if (CUT) { zt = cut_below(zt, cut_t); zd = cut_below(zd, cut_d); }
        const float p = pt.p(zt);
        acc_t += (double)p;
        acc_r += (double)fmaxf(0.f, p - pd.p(zd));
      });
    } else {
      visit_range<DT, false, 4>(row_t, nullptr, v0, v1, [&](int, float zt, float) {
        if (CUT) zt = cut_below(zt, cut_t);
        acc_t += (double)pt.p(zt);
      });
    }
  }
  *mass_r = block_sum_f64(acc_r, red);
  *mass_t = block_sum_f64(acc_t, red);
}

struct MassShared {
  BlockScratch red;
  Plan plan;
};

// grid (chunks, B): the accept decision of the sequence (every workgroup forms it for
// itself, chunk 0 publishes it), then the residual and target mass of one chunk of the
// sampling row.
template <int DT, bool CUT, bool CHAIN>
__global__ __launch_bounds__(kSampleThreads, 8) void verify_mass_kernel(VerifyArgs a) {
  __shared__ MassShared sh;
  const int b = blockIdx.y, c = blockIdx.x, C = gridDim.x;
  const int tid = threadIdx.x;
  SV_PHASE_MARK(6)
  if (tid < kWave) accept_plan<DT, CHAIN>(a, b, tid, c == 0, &sh.plan);
  __syncthreads();
  SV_PHASE_MARK(7)
  const Plan pl = sh.plan;
  double mass_r, mass_t;
  chunk_masses<DT, CUT>(a, b, pl, c, sh.red, &mass_r, &mass_t);
  SV_PHASE_MARK(8)
  if (tid == 0) {
    a.ws.mass_r[b * C + c] = mass_r;
    a.ws.mass_t[b * C + c] = mass_t;
  }
  SV_PHASE_MARK(9)
}

template <int THREADS>
struct PickShared {
  static constexpr int kSegT = kChunk / THREADS;      // contiguous weights per thread in the final scan
  BlockScratch red;
  union {
    float w[kChunk + kChunk / kSegT];  // weights of the located chunk (skewed)
    double mass[2 * kMaxChunks];     // before that: residual / target mass of every chunk
  };
  uint32_t flags;
  int chunk;
  int use_resid;
  int found_thread;
  double tau_local;
  double W;
};

// The token of sequence b from the chunk masses in sh.mass ([0, C) residual, [C, 2C) target;
// filled and visible to the whole workgroup of THREADS lanes): locate the chunk holding
// u' * W, stage its weights in LDS and find the token with a block prefix scan.
template <int DT, bool CUT, int THREADS>
__device__ __forceinline__ void pick_token(const VerifyArgs& a, const int b, const Plan& pl, PickShared<THREADS>& sh,
                                           const int C) {
  constexpr int kSegT = PickShared<THREADS>::kSegT;
  static_assert(sizeof(double) * 2 * kMaxChunks <= sizeof(float) * (kChunk + kChunk / kSegT), "mass fits under w");
  auto skew = [](int p) { return p + p / kSegT; };     // one padding word per segment: segment walks hit different banks
  const int tid = threadIdx.x;
  const int k = a.k, V = a.V;
  const int n = pl.n;
  const bool target_ok = pl.target_ok != 0;
  const bool resid = pl.resid != 0;
  const void* row_t = target_row<DT>(a, b, n);
  const void* row_d = resid ? draft_row<DT>(a, b, n) : nullptr;
  ProbRow pt, pd;
  pt.set(target_ok ? pl.lse_t : 0.0, a.sc_t);
  pd.set(resid ? pl.lse_d : 0.0, a.sc_d);
  float cut_t = -INFINITY, cut_d = -INFINITY;
  if (CUT) { cut_t = target_cut(a, b, n); if (resid) cut_d = draft_cut(a, b, n); }
  if (tid == 0) {
    uint32_t flags = pl.flags;
    const double* mr = sh.mass;
    const double* mt = sh.mass + C;
    double Wr = 0.0, Wt = 0.0;
    for (int j = 0; j < C; ++j) { Wr += mr[j]; Wt += mt[j]; }
    int use_resid = resid;
    // a residual of any mass is drawn from; only one without mass (or a non-finite one) is not
    if (target_ok && resid && !(isfinite(Wr) && Wr > 0.0)) { use_resid = 0; flags |= SV_FLAG_RESIDUAL_FALLBACK; }
    const double W = use_resid ? Wr : Wt;
    int chunk = -1;
    double tau_local = 0.0;
    if (target_ok && isfinite(W) && W > 0.0) {
      const U4 r = philox4x32_10((uint32_t)n, (uint32_t)b, 0u, a.step, a.seed_lo, a.seed_hi);
      const double tau = unit_from_word(r.w[1]) * W;
      const double* ms = use_resid ? mr : mt;
      double excl = 0.0;
      int last_pos = -1;
      double last_excl = 0.0;
      for (int j = 0; j < C; ++j) {
        const double mj = ms[j];
        if (mj > 0.0) { last_pos = j; last_excl = excl; }
        if (excl + mj > tau) { chunk = j; tau_local = tau - excl; break; }
        excl += mj;
      }
      if (chunk < 0) { chunk = last_pos; tau_local = tau - last_excl; }   // rounding: last chunk with mass
    } else {
      flags |= SV_FLAG_BAD_ROW;
    }
    sh.chunk = chunk;
    sh.tau_local = tau_local;
    sh.use_resid = use_resid;
    sh.W = W;
    sh.flags = flags;
    sh.found_thread = THREADS;
  }
  __syncthreads();
  SV_PHASE_MARK(2)
  const int chunk = sh.chunk;
  const int use_resid = sh.use_resid;
  int32_t* out = a.out_tokens + (size_t)b * (k + 1);
  if (chunk < 0) {                                     // nothing can be drawn
    if (tid == 0) a.flags[b] = sh.flags;
    return;
  }
  __syncthreads();                                     // masses are dead: w may overwrite them

  // stage the chunk's weights in LDS in vocabulary order
  const int w0 = chunk * kChunk, w1 = min(V, w0 + kChunk);
  for (int j = (w1 - w0) + tid; j < kChunk; j += THREADS) sh.w[skew(j)] = 0.f;
  if (use_resid) {
    visit_range<DT, true, 4>(row_t, row_d, w0, w1, [&](int v, float zt, float zd) {
      if (CUT) { zt = cut_below(zt, cut_t); zd = cut_below(zd, cut_d); }
      sh.w[skew(v - w0)] = fmaxf(0.f, pt.p(zt) - pd.p(zd));
    });
  } else {
    visit_range<DT, false, 4>(row_t, nullptr, w0, w1, [&](int v, float zt, float) {
      if (CUT) zt = cut_below(zt, cut_t);
      sh.w[skew(v - w0)] = pt.p(zt);
    });
  }
  __syncthreads();
  SV_PHASE_MARK(3)

  // block prefix scan over contiguous per-thread segments (fp64)
  static_assert(kSegT * THREADS == kChunk && (kSegT & (kSegT - 1)) == 0, "one segment per thread");
  const float* wseg = sh.w + tid * (kSegT + 1);         // this thread's segment, skewed
  double seg_sum = 0.0;
#pragma unroll 8
  for (int j = 0; j < kSegT; ++j) seg_sum += (double)wseg[j];
  // inclusive scan inside the wavefront, then across wavefronts through LDS
  double incl = seg_sum;
  const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int lo = __double2loint(incl), hi = __double2hiint(incl);
    lo = __shfl_up(lo, off, kWave);
    hi = __shfl_up(hi, off, kWave);
    const double o = __hiloint2double(hi, lo);
    if (lane >= off) incl += o;
  }
  if (lane == 63) sh.red.d[wave] = incl;
  __syncthreads();
  double wave_base = 0.0;
  for (int w = 0; w < wave; ++w) wave_base += sh.red.d[w];
  incl += wave_base;
  const double excl = incl - seg_sum;
  const double tau_local = sh.tau_local;
  // first thread whose inclusive sum passes the threshold; none when rounding
  // between the two passes put the threshold at or beyond the chunk total
  if (incl > tau_local) atomicMin(&sh.found_thread, tid);
  __syncthreads();
  SV_PHASE_MARK(4)
  int owner = sh.found_thread;
  const bool beyond = owner >= THREADS;
  if (beyond) owner = THREADS - 1;
  if (tid != owner) return;

  const double W = sh.W;
  double run = excl, prev = excl;
  int y = -1;
  if (!beyond) {
    for (int j = 0; j < kSegT; ++j) {
      prev = run;
      run += (double)wseg[j];
      if (run > tau_local) { y = tid * kSegT + j; break; }
    }
  }
  uint32_t fl = sh.flags;
  if (y >= 0) {
    if (fmin(run - tau_local, tau_local - prev) < kCdfEdgeRel * W + kCdfEdgeAbs) fl |= SV_FLAG_NEAR_CDF_EDGE;
  } else {
    // rounding left no entry whose running sum passes the threshold: take the
    // last positive-weight entry at or before the end of this segment
    fl |= SV_FLAG_NEAR_CDF_EDGE;
    for (int p = (tid + 1) * kSegT - 1; p >= 0; --p)
      if (sh.w[skew(p)] > 0.f) { y = p; break; }
  }
  if (y >= 0) out[n] = w0 + y; else fl |= SV_FLAG_BAD_ROW;   // y < 0: the chunk holds no mass at all
  a.flags[b] = fl;
}

// grid (B): the chunk masses of the sequence from the workspace, then the token.
template <int DT, bool CUT>
__global__ __launch_bounds__(kPickThreads) void verify_pick_kernel(VerifyArgs a, int C) {
  __shared__ PickShared<kPickThreads> sh;
  SV_PHASE_MARK(0)
  const int b = blockIdx.x;
  const Plan pl = a.ws.plan[b];
  for (int j = threadIdx.x; j < C; j += kPickThreads) {          // all chunk masses in one round of loads
    sh.mass[j] = a.ws.mass_r[(size_t)b * C + j];
    sh.mass[C + j] = a.ws.mass_t[(size_t)b * C + j];
  }
  __syncthreads();
  SV_PHASE_MARK(1)
  pick_token<DT, CUT, kPickThreads>(a, b, pl, sh, C);
  SV_PHASE_MARK(5)
}

// Workgroups per row: enough of them to spread the rows evenly over the CUs
// (1088 rows on 256 CUs leave some CUs a fifth more work than others) and to keep
// small batches from leaving CUs idle, but never parts shorter than 4096 entries.
// Measured at the five workloads: flat within 2 % from 3 to 8 workgroups per row.
static int rows_split(int rows, int V) {
  int s = (8192 + rows - 1) / rows;
  s = std::min(s, std::max(1, V / 4096));
  return std::max(1, std::min(s, kMaxSplit));
}

template <int DT, bool CUT>
static int launch_verify(const VerifyArgs& a, hipStream_t st) {
  const int rows = a.B * (a.chained ? a.k + 1 : 2 * a.k + 1);
  {
    TapScope tap(SV_KERNEL_VERIFY_ROWS, st);
    hipLaunchKernelGGL((verify_rows_kernel<DT, CUT>), dim3(rows * a.split), dim3(kRowsThreads), 0, st, a);
  }
  if (launch_status() != SV_OK) return SV_ERR_LAUNCH;
  const int C = n_chunks(a.V);
  {
    TapScope tap(SV_KERNEL_VERIFY_MASS, st);
    if (a.chained) hipLaunchKernelGGL((verify_mass_kernel<DT, CUT, true>), dim3(C, a.B), dim3(kSampleThreads), 0, st, a);
    else hipLaunchKernelGGL((verify_mass_kernel<DT, CUT, false>), dim3(C, a.B), dim3(kSampleThreads), 0, st, a);
  }
  if (launch_status() != SV_OK) return SV_ERR_LAUNCH;
  {
    TapScope tap(SV_KERNEL_VERIFY_PICK, st);
    hipLaunchKernelGGL((verify_pick_kernel<DT, CUT>), dim3(a.B), dim3(kPickThreads), 0, st, a, C);
  }
  return launch_status();
}

// Argument checks and launch shared by sv_verify_sample (T = 1, no cutoffs)
// and sv_verify_sample_warped.
static int verify_sample_checked(const void* z_t, const int32_t* t_offsets, int n_t_rows, const void* z_d,
                                 const int32_t* x, const int32_t* gamma, int B, int k, int V, int dtype,
                                 const Scale& sc_t, const float* cut_t, const Scale& sc_d, const float* cut_d,
                                 uint64_t seed, uint32_t step, int32_t* out_tokens, int32_t* n_accept,
                                 uint32_t* flags, float* ratio, void* ws, size_t ws_bytes, sv_stream_t stream,
                                 bool chained = false) {
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE(k <= SV_MAX_K && n_chunks(V) <= kMaxChunks, SV_ERR_TOO_LARGE);
  SV_REQUIRE((long long)B * (2 * k + 1) * kMaxSplit <= 0x7fffffffLL && B <= 65535, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(z_t && z_d && x && out_tokens && n_accept && flags, SV_ERR_NULL);
  SV_REQUIRE(!t_offsets || n_t_rows >= 0, SV_ERR_INVALID_ARG);
  const int eb = elem_bytes(dtype);
  SV_REQUIRE(is_aligned(z_t, eb) && is_aligned(z_d, eb), SV_ERR_ALIGN);
  SV_REQUIRE(is_aligned(x, 4) && is_aligned(out_tokens, 4) && is_aligned(n_accept, 4) &&
                 is_aligned(flags, 4) && is_aligned(t_offsets, 4) && is_aligned(gamma, 4) &&
                 is_aligned(ratio, 4) && is_aligned(cut_t, 4) && is_aligned(cut_d, 4),
             SV_ERR_ALIGN);
  SV_REQUIRE(ws && is_aligned(ws, kWsAlign) && ws_bytes >= sv_workspace_bytes(B, k, V, dtype),
             SV_ERR_WORKSPACE);
  VerifyArgs a;
  a.z_t = z_t; a.t_offsets = t_offsets; a.n_t_rows = n_t_rows;
  a.z_d = z_d; a.x = x; a.gamma = gamma;
  a.B = B; a.k = k; a.V = V;
  a.chained = chained ? 1 : 0;
  a.dtype = dtype;
  a.split = rows_split(B * (chained ? k + 1 : 2 * k + 1), V);
  a.t_seq_rows = k + 1;
  a.with_bonus = 1;
  a.seed_lo = (uint32_t)(seed & 0xffffffffu); a.seed_hi = (uint32_t)(seed >> 32); a.step = step;
  a.out_tokens = out_tokens; a.n_accept = n_accept; a.flags = flags; a.ratio = ratio;
  a.sc_t = sc_t; a.sc_d = sc_d; a.cut_t = cut_t; a.cut_d = cut_d;
  a.ws = carve_verify_ws(ws, B, k, V);
  hipStream_t st = as_stream(stream);
  if (cut_t || cut_d)
    return dtype == SV_F32 ? launch_verify<DT_F32, true>(a, st) : launch_verify<DT_BF16, true>(a, st);
  return dtype == SV_F32 ? launch_verify<DT_F32, false>(a, st) : launch_verify<DT_BF16, false>(a, st);
}

// ---------------------------------------------------------------------------
// Scratch of the entry point that takes no workspace: one array per GPU, held
// until the process ends.  In host code the array's name is only a stand-in;
// the address on the current device comes from hipGetSymbolAddress, once per
// device, and only that pointer is ever handed to a kernel.
// ---------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[SV_STATIC_SCRATCH_BYTES];

static int static_scratch(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr_of[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SV_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr_of[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SV_ERR_LAUNCH;
    ptr_of[dev] = p;
  }
  *out = ptr_of[dev];
  return SV_OK;
}

}  // namespace sv

extern "C" int sv_verify_sample_static(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                                       const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                                       int B, int k, int V, int dtype, uint64_t seed, uint32_t step,
                                       int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                                       float* ratio_or_null, sv_stream_t stream) {
  using namespace sv;
  // sizes first, so that a shape beyond the scratch is told apart from other errors
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE(k <= SV_MAX_K && n_chunks(V) <= kMaxChunks, SV_ERR_TOO_LARGE);
  SV_REQUIRE((long long)B * (2 * k + 1) * kMaxSplit <= 0x7fffffffLL && B <= 65535, SV_ERR_TOO_LARGE);
  SV_REQUIRE(sv_workspace_bytes(B, k, V, dtype) <= (size_t)SV_STATIC_SCRATCH_BYTES, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  void* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != SV_OK) return rc;
  return verify_sample_checked(z_t, t_offsets_or_null, n_t_rows, z_d, x, gamma_or_null, B, k, V, dtype,
                               unit_scale(), nullptr, unit_scale(), nullptr, seed, step, out_tokens, n_accept,
                               flags, ratio_or_null, ws, SV_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int sv_verify_sample(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                                const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                                int B, int k, int V, int dtype, uint64_t seed, uint32_t step,
                                int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                                float* ratio_or_null, void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  return verify_sample_checked(z_t, t_offsets_or_null, n_t_rows, z_d, x, gamma_or_null, B, k, V, dtype,
                               unit_scale(), nullptr, unit_scale(), nullptr, seed, step, out_tokens, n_accept,
                               flags, ratio_or_null, ws, ws_bytes, stream);
}

extern "C" int sv_verify_sample_warped(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                                       const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                                       int B, int k, int V, int dtype,
                                       float temperature_t, const float* cutoff_t_or_null,
                                       float temperature_d, const float* cutoff_d_or_null,
                                       uint64_t seed, uint32_t step,
                                       int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                                       float* ratio_or_null, void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  Scale sc_t, sc_d;
  SV_REQUIRE(scale_of(temperature_t, &sc_t) && scale_of(temperature_d, &sc_d), SV_ERR_INVALID_ARG);
  return verify_sample_checked(z_t, t_offsets_or_null, n_t_rows, z_d, x, gamma_or_null, B, k, V, dtype,
                               sc_t, cutoff_t_or_null, sc_d, cutoff_d_or_null, seed, step, out_tokens, n_accept,
                               flags, ratio_or_null, ws, ws_bytes, stream);
}

extern "C" int sv_verify_sample_chained(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                                        const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                                        int B, int k, int V, int dtype, uint64_t seed, uint32_t step,
                                        int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                                        float* ratio_or_null, void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  return verify_sample_checked(z_t, t_offsets_or_null, n_t_rows, z_d, x, gamma_or_null, B, k, V, dtype,
                               unit_scale(), nullptr, unit_scale(), nullptr, seed, step, out_tokens, n_accept,
                               flags, ratio_or_null, ws, ws_bytes, stream, true);
}

extern "C" int sv_verify_sample_warped_chained(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                                               const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                                               int B, int k, int V, int dtype,
                                               float temperature_t, const float* cutoff_t_or_null,
                                               float temperature_d, const float* cutoff_d_or_null,
                                               uint64_t seed, uint32_t step,
                                               int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                                               float* ratio_or_null, void* ws, size_t ws_bytes,
                                               sv_stream_t stream) {
  using namespace sv;
  Scale sc_t, sc_d;
  SV_REQUIRE(scale_of(temperature_t, &sc_t) && scale_of(temperature_d, &sc_d), SV_ERR_INVALID_ARG);
  return verify_sample_checked(z_t, t_offsets_or_null, n_t_rows, z_d, x, gamma_or_null, B, k, V, dtype,
                               sc_t, cutoff_t_or_null, sc_d, cutoff_d_or_null, seed, step, out_tokens, n_accept,
                               flags, ratio_or_null, ws, ws_bytes, stream, true);
}

namespace sv {
// Argument checks and launch shared by sv_accept_ratio (T = 1, no cutoffs) and
// sv_accept_ratio_warped.
static int accept_ratio_checked(const void* z_t, int t_rows_per_seq, const void* z_d, const int32_t* x,
                                int B, int k, int V, int dtype, const Scale& sc_t, const float* cut_t,
                                const Scale& sc_d, const float* cut_d, float* ratio, uint32_t* flags,
                                void* ws, size_t ws_bytes, sv_stream_t stream) {
  SV_REQUIRE(dtype == SV_F32 || dtype == SV_BF16, SV_ERR_DTYPE);
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE(t_rows_per_seq == k || t_rows_per_seq == k + 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE((long long)B * (2 * k + 1) * kMaxSplit <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(z_t && z_d && x && ratio, SV_ERR_NULL);
  const int eb = elem_bytes(dtype);
  SV_REQUIRE(is_aligned(z_t, eb) && is_aligned(z_d, eb) && is_aligned(x, 4) && is_aligned(ratio, 4) &&
                 is_aligned(flags, 4) && is_aligned(cut_t, 4) && is_aligned(cut_d, 4),
             SV_ERR_ALIGN);
  SV_REQUIRE(ws && is_aligned(ws, kWsAlign) && ws_bytes >= sv_workspace_bytes(B, k, V, dtype),
             SV_ERR_WORKSPACE);
  VerifyArgs a = {};
  a.z_t = z_t; a.t_offsets = nullptr; a.n_t_rows = 0;
  a.z_d = z_d; a.x = x; a.gamma = nullptr;
  a.B = B; a.k = k; a.V = V;
  a.split = rows_split(B * 2 * k, V);
  a.t_seq_rows = t_rows_per_seq;
  a.with_bonus = 0;
  a.sc_t = sc_t; a.sc_d = sc_d; a.cut_t = cut_t; a.cut_d = cut_d;
  a.ws = carve_verify_ws(ws, B, k, V);
  hipStream_t st = as_stream(stream);
  const int rows = B * (2 * k + 1);               // the bonus slots exit at once
  const bool cut = cut_t || cut_d;
  {
    TapScope tap(SV_KERNEL_VERIFY_ROWS, st);
    const dim3 grid(rows * a.split), block(kRowsThreads);
    if (dtype == SV_F32) {
      if (cut) hipLaunchKernelGGL((verify_rows_kernel<DT_F32, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((verify_rows_kernel<DT_F32, false>), grid, block, 0, st, a);
    } else {
      if (cut) hipLaunchKernelGGL((verify_rows_kernel<DT_BF16, true>), grid, block, 0, st, a);
      else hipLaunchKernelGGL((verify_rows_kernel<DT_BF16, false>), grid, block, 0, st, a);
    }
  }
  if (launch_status() != SV_OK) return SV_ERR_LAUNCH;
  hipLaunchKernelGGL(accept_ratio_kernel, dim3(B), dim3(kWave), 0, st, a, ratio, flags);
  return launch_status();
}
}  // namespace sv

extern "C" int sv_accept_ratio(const void* z_t, int t_rows_per_seq, const void* z_d, const int32_t* x,
                               int B, int k, int V, int dtype, float* ratio, uint32_t* flags_or_null,
                               void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  return accept_ratio_checked(z_t, t_rows_per_seq, z_d, x, B, k, V, dtype, unit_scale(), nullptr, unit_scale(),
                              nullptr, ratio, flags_or_null, ws, ws_bytes, stream);
}

extern "C" int sv_accept_ratio_warped(const void* z_t, int t_rows_per_seq, const void* z_d, const int32_t* x,
                                      int B, int k, int V, int dtype,
                                      float temperature_t, const float* cutoff_t_or_null,
                                      float temperature_d, const float* cutoff_d_or_null,
                                      float* ratio, uint32_t* flags_or_null,
                                      void* ws, size_t ws_bytes, sv_stream_t stream) {
  using namespace sv;
  Scale sc_t, sc_d;
  SV_REQUIRE(scale_of(temperature_t, &sc_t) && scale_of(temperature_d, &sc_d), SV_ERR_INVALID_ARG);
  return accept_ratio_checked(z_t, t_rows_per_seq, z_d, x, B, k, V, dtype, sc_t, cutoff_t_or_null, sc_d,
                              cutoff_d_or_null, ratio, flags_or_null, ws, ws_bytes, stream);
}
