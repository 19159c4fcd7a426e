// sv_row_stats_sparse / sv_verify_sample_sparse: the SV indicators (Sec. 4.2 and
// the appendix definitions of S and A) and speculative-sampling verification
// on the compacted supports written by sv_warp_compact.  With the sampling
// hyper-parameters of the paper's appendix table a warped distribution lives on
// a few dozen tokens, so every quantity here is a sum over two short, sorted
// token lists; all arithmetic is fp64 and one wavefront handles one (sequence,
// position) pair or one sequence.  Launch-latency bound.
#include "sv_device.hpp"
#include "sv_host.hpp"

namespace sv {

// One tensor's supports: row r owns token[r*cap .. r*cap + count[r]) (ascending ids).
struct Supports {
  const int32_t* count;
  const int32_t* token;
  const double* prob;
  int cap;
};

// Probability of token t in a row's support (0 when it is not listed).
__device__ __forceinline__ double support_prob(const Supports& s, long row, int n, int t) {
  const int32_t* tok = s.token + row * s.cap;
  int lo = 0, hi = n;                       // first index with tok[idx] >= t
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (tok[mid] < t) lo = mid + 1; else hi = mid;
  }
  return (lo < n && tok[lo] == t) ? s.prob[row * s.cap + lo] : 0.0;
}

struct SparseStatsArgs {
  Supports d, c;
  const float* lse_d_in;
  const float* lse_c_in;
  const int32_t* x;
  int pairs, V;
  float* lse_d;
  float* lse_c;
  float* S;
  float* A;
  float* kl;          // nullable
  float* entropy_d;   // nullable
  float* pd_x;        // nullable
  uint32_t* flags;    // nullable
};

constexpr int kSparseStatsWaves = 4;

// one wavefront per (sequence, position)
__global__ __launch_bounds__(kSparseStatsWaves* kWave) void row_stats_sparse_kernel(SparseStatsArgs a) {
  const int pair = blockIdx.x * kSparseStatsWaves + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (pair >= a.pairs) return;
  const int nd = a.d.count[pair], nc = a.c.count[pair];
  uint32_t fl = 0;
  if (nd < 0 || nc < 0) fl |= SV_FLAG_NOT_COMPACT;
  else if (nd == 0 || nc == 0) fl |= SV_FLAG_BAD_ROW;
  const double nan = __builtin_nan("");
  double S = nan, KL = nan, H = nan, A = nan, pdx = nan;
  if (!fl) {
    double s = 0.0, kl = 0.0, h = 0.0;
    for (int j = lane; j < nd; j += kWave) {
      const double pd = a.d.prob[(long)pair * a.d.cap + j];
      const double pc = support_prob(a.c, pair, nc, a.d.token[(long)pair * a.d.cap + j]);
      s += fmin(pd, pc);
      const double lpd = log(pd);
      kl += pd * (lpd - log(pc));           // +inf where the companion's support misses the token
      h -= pd * lpd;
    }
    S = wave_sum_f64(s);
    KL = wave_sum_f64(kl);
    H = wave_sum_f64(h);
    const int tok = a.x[pair];
    if (tok < 0 || tok >= a.V) {
      fl |= SV_FLAG_BAD_TOKEN;
    } else {
      pdx = support_prob(a.d, pair, nd, tok);
      const double pcx = support_prob(a.c, pair, nc, tok);
      A = (pdx == 0.0) ? 1.0 : fmin(1.0, pcx / pdx);
    }
  }
  if (lane == 0) {
    const bool valid = !(fl & (SV_FLAG_NOT_COMPACT | SV_FLAG_BAD_ROW));
    a.lse_d[pair] = valid ? a.lse_d_in[pair] : __builtin_nanf("");
    a.lse_c[pair] = valid ? a.lse_c_in[pair] : __builtin_nanf("");
    a.S[pair] = (float)S;
    a.A[pair] = (float)A;
    if (a.kl) a.kl[pair] = (float)KL;
    if (a.entropy_d) a.entropy_d[pair] = (float)H;
    if (a.pd_x) a.pd_x[pair] = (float)pdx;
    if (a.flags) a.flags[pair] = fl;
  }
}

struct SparseVerifyArgs {
  Supports t, d;
  const int32_t* t_offsets;   // nullable
  int n_t_rows;
  const int32_t* x;
  const int32_t* gamma;       // nullable
  int B, k, V;
  uint32_t seed_lo, seed_hi, step;
  int32_t* out_tokens;
  int32_t* n_accept;
  uint32_t* flags;
  float* ratio;               // nullable
};

__device__ __forceinline__ long sparse_target_index(const SparseVerifyArgs& a, int b, int i) {
  if (a.t_offsets) {
    const long row = (long)a.t_offsets[b] + i;
    return (row < 0 || row >= a.n_t_rows) ? -1 : row;
  }
  return (long)b * (a.k + 1) + i;
}

// Sampling weight of entry j of the target support of row `trow`.
__device__ __forceinline__ double sample_weight(const SparseVerifyArgs& a, long trow, int j, bool resid, long drow,
                                                int nd) {
  const double pt = a.t.prob[trow * a.t.cap + j];
  if (!resid) return pt;
  return fmax(0.0, pt - support_prob(a.d, drow, nd, a.t.token[trow * a.t.cap + j]));
}

// one wavefront per sequence; lane i evaluates drafted position i (k <= 64)
__global__ __launch_bounds__(kWave) void verify_sample_sparse_kernel(SparseVerifyArgs a) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const int k = a.k;
  int g = a.gamma ? a.gamma[b] : k;
  g = min(max(g, 0), k);
  const bool evaluated = lane < g;
  bool accept = true;
  uint32_t fl = 0;
  double rho = __builtin_nan("");
  if (evaluated) {
    const int tok = a.x[b * k + lane];
    const long trow = sparse_target_index(a, b, lane);
    const long drow = (long)b * k + lane;
    const int nt = trow >= 0 ? a.t.count[trow] : 0;
    const int nd = a.d.count[drow];
    if (tok < 0 || tok >= a.V) {
      fl |= SV_FLAG_BAD_TOKEN;
    } else if (nt < 0 || nd < 0) {
      fl |= SV_FLAG_NOT_COMPACT | SV_FLAG_BAD_ROW;
    } else if (nt == 0 || nd == 0) {
      fl |= SV_FLAG_BAD_ROW;
    } else {
      const double pt = support_prob(a.t, trow, nt, tok), pd = support_prob(a.d, drow, nd, tok);
      rho = pt / pd;                              // 0/0 = NaN: rejected; p/0 = +inf: accepted
    }
    const U4 r = philox4x32_10((uint32_t)lane, (uint32_t)b, 0u, a.step, a.seed_lo, a.seed_hi);
    const double u = unit_from_word(r.w[0]);
    accept = u < rho;                             // false for NaN
    if (!isnan(rho) && fabs(u - fmin(1.0, rho)) < 1e-6) fl |= SV_FLAG_NEAR_TIE;
  }
  const unsigned long long rej = __ballot(evaluated && !accept);
  const int n = rej ? (int)__builtin_ctzll(rej) : g;          // leading accepts
  if (!(evaluated && lane <= n)) fl = 0;                        // flags of the positions actually evaluated
  for (int off = 32; off >= 1; off >>= 1) fl |= __shfl_xor(fl, off, kWave);
  if (a.ratio && lane < k) a.ratio[b * k + lane] = (evaluated && lane <= n) ? (float)rho : __builtin_nanf("");
  int32_t* out = a.out_tokens + (size_t)b * (k + 1);
  for (int j = lane; j <= k; j += kWave) out[j] = (j < n) ? a.x[b * k + j] : -1;

  // ---- the token of position n: residual after a rejection, target row otherwise
  const long trow = sparse_target_index(a, b, n);
  const int nt = trow >= 0 ? a.t.count[trow] : 0;
  bool resid = n < g;
  long drow = 0;
  int nd = 0;
  if (resid) {
    drow = (long)b * k + n;
    nd = a.d.count[drow];
    if (nd <= 0) {                                // unusable draft row: draw from the target instead
      resid = false;
      fl |= SV_FLAG_BAD_ROW | SV_FLAG_RESIDUAL_FALLBACK | (nd < 0 ? SV_FLAG_NOT_COMPACT : 0u);
    }
  }
  if (nt <= 0) {
    fl |= SV_FLAG_BAD_ROW | (nt < 0 ? SV_FLAG_NOT_COMPACT : 0u);
    if (lane == 0) { a.flags[b] = fl; a.n_accept[b] = n; }
    return;
  }
  const int seg = (nt + kWave - 1) / kWave;       // contiguous entries per lane
  const int j0 = min(lane * seg, nt), j1 = min(j0 + seg, nt);
  double part = 0.0;
  for (int j = j0; j < j1; ++j) part += sample_weight(a, trow, j, resid, drow, nd);
  double W = wave_sum_f64(part);
  if (resid && !(isfinite(W) && W > 0.0)) {   // residual without mass: draw from the target
    resid = false;
    fl |= SV_FLAG_RESIDUAL_FALLBACK;
    part = 0.0;
    for (int j = j0; j < j1; ++j) part += sample_weight(a, trow, j, false, drow, nd);
    W = wave_sum_f64(part);
  }
  if (!(isfinite(W) && W > 0.0)) {
    if (lane == 0) { a.flags[b] = fl | SV_FLAG_BAD_ROW; a.n_accept[b] = n; }
    return;
  }
  const U4 r = philox4x32_10((uint32_t)n, (uint32_t)b, 0u, a.step, a.seed_lo, a.seed_hi);
  const double tau = unit_from_word(r.w[1]) * W;
  double incl = part;                              // inclusive scan of the segment sums
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    int lo = __double2loint(incl), hi = __double2hiint(incl);
    lo = __shfl_up(lo, off, kWave);
    hi = __shfl_up(hi, off, kWave);
    const double o = __hiloint2double(hi, lo);
    if (lane >= off) incl += o;
  }
  const unsigned long long pass = __ballot(incl > tau && j1 > j0);
  int owner = pass ? (int)__builtin_ctzll(pass) : -1;
  if (owner < 0) {
    // rounding left the threshold at or beyond the total: the last lane that owns entries decides
    const unsigned long long has = __ballot(j1 > j0);
    owner = 63 - (int)__builtin_clzll(has);
  }
  if (lane == owner) {
    double run = incl - part, prev = run;
    int y = -1;
    if (pass) {
      for (int j = j0; j < j1; ++j) {
        prev = run;
        run += sample_weight(a, trow, j, resid, drow, nd);
        if (run > tau) { y = j; break; }
      }
    }
    if (y >= 0) {
      if (fmin(run - tau, tau - prev) < kCdfEdgeRel * W) fl |= SV_FLAG_NEAR_CDF_EDGE;
    } else {
      fl |= SV_FLAG_NEAR_CDF_EDGE;               // take the last entry that carries weight
      for (int j = j1 - 1; j >= 0; --j)
        if (sample_weight(a, trow, j, resid, drow, nd) > 0.0) { y = j; break; }
    }
    if (y >= 0) out[n] = a.t.token[trow * a.t.cap + y]; else fl |= SV_FLAG_BAD_ROW;
    a.flags[b] = fl;
    a.n_accept[b] = n;
  }
}

// one lane per (sequence, position): p_t(x) / p_d(x) of every drafted position (profile
// construction: no early stop, no sampling)
__global__ void accept_ratio_sparse_kernel(Supports t, Supports d, int t_rows_per_seq, const int32_t* x, int B,
                                           int k, int V, float* ratio, uint32_t* flags) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= B * k) return;
  const int b = j / k, i = j - b * k;
  const long trow = (long)b * t_rows_per_seq + i, drow = j;
  const int tok = x[j], nt = t.count[trow], nd = d.count[drow];
  uint32_t fl = 0;
  double rho = __builtin_nan("");
  if (tok < 0 || tok >= V) fl |= SV_FLAG_BAD_TOKEN;
  else if (nt < 0 || nd < 0) fl |= SV_FLAG_NOT_COMPACT;
  else if (nt == 0 || nd == 0) fl |= SV_FLAG_BAD_ROW;
  else rho = support_prob(t, trow, nt, tok) / support_prob(d, drow, nd, tok);
  ratio[j] = (float)rho;
  if (flags) flags[j] = fl;
}

}  // namespace sv

extern "C" int sv_row_stats_sparse(const int32_t* count_d, const int32_t* token_d, const double* prob_d,
                                   const float* lse_d_in, const int32_t* count_c, const int32_t* token_c,
                                   const double* prob_c, const float* lse_c_in, int cap, const int32_t* x,
                                   int B, int k, int V, float* lse_d, float* lse_c, float* S, float* A,
                                   float* kl_or_null, float* entropy_d_or_null, float* pd_x_or_null,
                                   uint32_t* flags_or_null, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1 && cap >= 1 && cap <= SV_SUPPORT_MAX_CAP, SV_ERR_INVALID_ARG);
  SV_REQUIRE((long long)B * k <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(count_d && token_d && prob_d && lse_d_in && count_c && token_c && prob_c && lse_c_in && x && lse_d &&
                 lse_c && S && A,
             SV_ERR_NULL);
  SV_REQUIRE(is_aligned(count_d, 4) && is_aligned(token_d, 4) && is_aligned(prob_d, 8) && is_aligned(lse_d_in, 4) &&
                 is_aligned(count_c, 4) && is_aligned(token_c, 4) && is_aligned(prob_c, 8) &&
                 is_aligned(lse_c_in, 4) && is_aligned(x, 4) && is_aligned(lse_d, 4) && is_aligned(lse_c, 4) &&
                 is_aligned(S, 4) && is_aligned(A, 4) && is_aligned(kl_or_null, 4) &&
                 is_aligned(entropy_d_or_null, 4) && is_aligned(pd_x_or_null, 4) && is_aligned(flags_or_null, 4),
             SV_ERR_ALIGN);
  SparseStatsArgs a;
  a.d = Supports{count_d, token_d, prob_d, cap};
  a.c = Supports{count_c, token_c, prob_c, cap};
  a.lse_d_in = lse_d_in; a.lse_c_in = lse_c_in; a.x = x; a.pairs = B * k; a.V = V;
  a.lse_d = lse_d; a.lse_c = lse_c; a.S = S; a.A = A; a.kl = kl_or_null; a.entropy_d = entropy_d_or_null;
  a.pd_x = pd_x_or_null; a.flags = flags_or_null;
  const int blocks = (a.pairs + kSparseStatsWaves - 1) / kSparseStatsWaves;
  hipLaunchKernelGGL(row_stats_sparse_kernel, dim3(blocks), dim3(kSparseStatsWaves * kWave), 0, as_stream(stream), a);
  return launch_status();
}

extern "C" int sv_verify_sample_sparse(const int32_t* count_t, const int32_t* token_t, const double* prob_t,
                                       const int32_t* t_offsets_or_null, int n_t_rows, const int32_t* count_d,
                                       const int32_t* token_d, const double* prob_d, int cap, const int32_t* x,
                                       const int32_t* gamma_or_null, int B, int k, int V, uint64_t seed,
                                       uint32_t step, int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                                       float* ratio_or_null, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1 && cap >= 1 && cap <= SV_SUPPORT_MAX_CAP, SV_ERR_INVALID_ARG);
  SV_REQUIRE(k <= SV_MAX_K, SV_ERR_TOO_LARGE);
  SV_REQUIRE((long long)B * (k + 1) <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(count_t && token_t && prob_t && count_d && token_d && prob_d && x && out_tokens && n_accept && flags,
             SV_ERR_NULL);
  SV_REQUIRE(!t_offsets_or_null || n_t_rows >= 0, SV_ERR_INVALID_ARG);
  SV_REQUIRE(is_aligned(count_t, 4) && is_aligned(token_t, 4) && is_aligned(prob_t, 8) && is_aligned(count_d, 4) &&
                 is_aligned(token_d, 4) && is_aligned(prob_d, 8) && is_aligned(x, 4) &&
                 is_aligned(t_offsets_or_null, 4) && is_aligned(gamma_or_null, 4) && is_aligned(out_tokens, 4) &&
                 is_aligned(n_accept, 4) && is_aligned(flags, 4) && is_aligned(ratio_or_null, 4),
             SV_ERR_ALIGN);
  SparseVerifyArgs a;
  a.t = Supports{count_t, token_t, prob_t, cap};
  a.d = Supports{count_d, token_d, prob_d, cap};
  a.t_offsets = t_offsets_or_null; a.n_t_rows = n_t_rows; a.x = x; a.gamma = gamma_or_null;
  a.B = B; a.k = k; a.V = V;
  a.seed_lo = (uint32_t)(seed & 0xffffffffu); a.seed_hi = (uint32_t)(seed >> 32); a.step = step;
  a.out_tokens = out_tokens; a.n_accept = n_accept; a.flags = flags; a.ratio = ratio_or_null;
  hipLaunchKernelGGL(verify_sample_sparse_kernel, dim3(B), dim3(kWave), 0, as_stream(stream), a);
  return launch_status();
}

extern "C" int sv_accept_ratio_sparse(const int32_t* count_t, const int32_t* token_t, const double* prob_t,
                                      int t_rows_per_seq, const int32_t* count_d, const int32_t* token_d,
                                      const double* prob_d, int cap, const int32_t* x, int B, int k, int V,
                                      float* ratio, uint32_t* flags_or_null, sv_stream_t stream) {
  using namespace sv;
  SV_REQUIRE(B >= 0 && k >= 1 && V >= 1 && cap >= 1 && cap <= SV_SUPPORT_MAX_CAP, SV_ERR_INVALID_ARG);
  SV_REQUIRE(t_rows_per_seq == k || t_rows_per_seq == k + 1, SV_ERR_INVALID_ARG);
  SV_REQUIRE((long long)B * (k + 1) <= 0x7fffffffLL, SV_ERR_TOO_LARGE);
  if (B == 0) return SV_OK;
  SV_REQUIRE(count_t && token_t && prob_t && count_d && token_d && prob_d && x && ratio, SV_ERR_NULL);
  SV_REQUIRE(is_aligned(count_t, 4) && is_aligned(token_t, 4) && is_aligned(prob_t, 8) && is_aligned(count_d, 4) &&
                 is_aligned(token_d, 4) && is_aligned(prob_d, 8) && is_aligned(x, 4) && is_aligned(ratio, 4) &&
                 is_aligned(flags_or_null, 4),
             SV_ERR_ALIGN);
  const int n = B * k, threads = 256;
  hipLaunchKernelGGL(accept_ratio_sparse_kernel, dim3((n + threads - 1) / threads), dim3(threads), 0,
                     as_stream(stream), Supports{count_t, token_t, prob_t, cap}, Supports{count_d, token_d, prob_d, cap},
                     t_rows_per_seq, x, B, k, V, ratio, flags_or_null);
  return launch_status();
}
